// lags_sparsify_layer_noalloc: Algorithm 1 lines 6-7 for one layer without any allocation.
//
// For callers that cannot call hipMalloc (code under HIP graph capture, tight serving loops,
// harnesses that forbid it).  Everything the kernels need beyond the caller's buffers (the
// one-layer plan, the candidate slots, counts and partial histograms) lives in one
// file-scope device array of kStaticBytes bytes.  Each GPU that the library runs on holds its
// own copy of that array until the process ends; its address on a device is looked up once per
// device with hipGetSymbolAddress and that pointer, never the array's name, is what host code
// passes on.  The array keeps the last call's contents; every call writes what it reads (the
// plan kernel writes the plan, the sample kernel resets the layer's state), so nothing has to
// be cleared between calls.  Calls that overlap in time on one GPU share the array and race.
#include "../../include/lags.h"
#include "lags_internal.h"

#include <cmath>
#include <mutex>

using namespace lags;

namespace {

constexpr int kStaticMaxTiles = 4096;                     // d <= 16,777,216
constexpr int64_t kStaticMaxSlots = 1 << 19;              // tiles x slots per tile (8 bytes each)
constexpr size_t kStaticBytes = 5u << 20;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

std::mutex g_mutex;
unsigned char* g_ptr[kMaxDevices] = {};   // per device: the address of its copy of `scratch`

struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
    if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
  }
  ~DeviceGuard() {
    int cur = -1;
    if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
  }
};

// Byte offsets of the parts of the array for the largest supported layer (all multiples of 256).
struct Layout {
  size_t segs, list, lseg, multi, tiles, groups, hparts;                       // the plan
  size_t lstate, chunk_cnt, slots, wgt, band, band_cnt, bh_part, coarse_part,  // per-call scratch
      part_info, ghist, dstate, tile_gt, tile_eq, items, fail, end;
};

constexpr size_t up256(size_t x) { return (x + 255) / 256 * 256; }

constexpr Layout make_layout() {
  Layout L = {};
  constexpr size_t nt = kStaticMaxTiles;
  constexpr size_t nwc = (nt + kWaveTiles - 1) / kWaveTiles;
  constexpr size_t ng = (nwc + kGroupWaves - 1) / kGroupWaves;
  constexpr size_t nh = (nt + kCountTiles - 1) / kCountTiles;
  size_t at = 0;
  L.segs = at; at = up256(at + sizeof(SegDesc));
  L.list = at; at = up256(at + sizeof(int32_t));
  L.lseg = at; at = up256(at + sizeof(LargeSeg));
  L.multi = at; at = up256(at + sizeof(int32_t));
  L.tiles = at; at = up256(at + nt * sizeof(TileDesc));
  L.groups = at; at = up256(at + ng * sizeof(GroupDesc));
  L.hparts = at; at = up256(at + nh * sizeof(GroupDesc));
  L.lstate = at; at = up256(at + sizeof(LState));
  L.chunk_cnt = at; at = up256(at + nt * sizeof(uint32_t));
  L.slots = at; at = up256(at + (size_t)kStaticMaxSlots * sizeof(uint2));
  L.wgt = at; at = up256(at + (nwc + 4) * sizeof(uint32_t));
  L.band = at; at = up256(at + ng * kGroupBand * sizeof(uint2));
  L.band_cnt = at; at = up256(at + ng * sizeof(uint32_t));
  L.bh_part = at; at = up256(at + nh * kFineBins * sizeof(uint32_t));
  L.coarse_part = at; at = up256(at + nh * kCoarseBins * sizeof(uint32_t));
  L.part_info = at; at = up256(at + nh * sizeof(uint4));
  L.ghist = at; at = up256(at + (kHistStride + 16) * sizeof(uint32_t));
  L.dstate = at; at = up256(at + sizeof(DState));
  L.tile_gt = at; at = up256(at + nt * sizeof(uint32_t));
  L.tile_eq = at; at = up256(at + nt * sizeof(uint32_t));
  L.items = at; at = up256(at + nt * sizeof(int32_t));
  L.fail = at; at = up256(at + sizeof(uint32_t));
  L.end = at;
  return L;
}

constexpr Layout kLayout = make_layout();
static_assert(kLayout.end <= kStaticBytes, "the static array holds the largest supported layer");

// The plan of one layer at offset 0, passed to the plan kernel by value.
struct OneLayer {
  int32_t d, k;
  int32_t n_tiles, n_groups, n_hparts;
  LargeSeg ls;
};

// Writes the one-layer plan into the array: the layer, its large-path plan and its tiles.
__global__ __launch_bounds__(256) void k_plan_layer(unsigned char* __restrict__ base, OneLayer p) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i == 0) {
    SegDesc sd;
    sd.offset = 0;
    sd.out_offset = 0;
    sd.d = p.d;
    sd.k = p.k;
    *reinterpret_cast<SegDesc*>(base + kLayout.segs) = sd;
    *reinterpret_cast<int32_t*>(base + kLayout.list) = 0;
    *reinterpret_cast<LargeSeg*>(base + kLayout.lseg) = p.ls;
    *reinterpret_cast<int32_t*>(base + kLayout.multi) = 0;
  }
  if (i < p.n_tiles) {
    TileDesc td;
    td.start = (int64_t)i * kTile;
    td.n = p.d - i * kTile < kTile ? p.d - i * kTile : kTile;
    td.seg = 0;
    td.local0 = i * kTile;
    td.ctile = p.ls.sampled ? i : -1;
    reinterpret_cast<TileDesc*>(base + kLayout.tiles)[i] = td;
  }
  if (i < p.n_groups) {
    GroupDesc gd;
    gd.lseg = 0;
    gd.first = i;
    reinterpret_cast<GroupDesc*>(base + kLayout.groups)[i] = gd;
  }
  if (i < p.n_hparts) {
    GroupDesc hp;
    hp.lseg = 0;
    hp.first = i;
    reinterpret_cast<GroupDesc*>(base + kLayout.hparts)[i] = hp;
  }
}

bool ranges_overlap(const void* a, int64_t abytes, const void* b, int64_t bbytes) {
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a0 < b0 + (uintptr_t)bbytes && b0 < a0 + (uintptr_t)abytes;
}

// The address of this device's copy of the array (looked up once per device, with that device current).
int device_scratch(int device, unsigned char** out) {
  std::lock_guard<std::mutex> lock(g_mutex);
  if (!g_ptr[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LAGS_EHIP;
    g_ptr[device] = static_cast<unsigned char*>(p);
  }
  *out = g_ptr[device];
  return LAGS_OK;
}

}  // namespace

extern "C" {

int64_t lags_noalloc_max_elements(void) { return (int64_t)kStaticMaxTiles * kTile; }

int lags_sparsify_layer_noalloc(int device, const float* grad, float* residual, int64_t d, float lr, int64_t k,
                                int32_t* out_idx, float* out_val, void* hip_stream) {
  if (!grad || !residual || !out_idx || !out_val) return LAGS_EINVAL;
  if (d < 1 || d > 0x7FFFFFFFLL || k < 1 || k > d || !std::isfinite(lr)) return LAGS_EINVAL;
  if (device < 0 || device >= kMaxDevices) return LAGS_EINVAL;
  const int64_t db = d * 4, kb = k * 4;
  if (ranges_overlap(grad, db, residual, db) || ranges_overlap(out_idx, kb, out_val, kb) ||
      ranges_overlap(grad, db, out_idx, kb) || ranges_overlap(grad, db, out_val, kb) ||
      ranges_overlap(residual, db, out_idx, kb) || ranges_overlap(residual, db, out_val, kb))
    return LAGS_EINVAL;
  if (d > lags_noalloc_max_elements()) return LAGS_ECAPACITY;
  // the plan, on the stack
  OneLayer p = {};
  p.d = (int32_t)d;
  p.k = (int32_t)k;
  const int cls = d <= kSmall0 ? 0 : (d <= kSmall1 ? 1 : kSmallClasses);
  LargePlan pl;
  if (cls == kSmallClasses) {
    const int64_t nt = (d + kTile - 1) / kTile;
    double per_tile = 0.0;
    LargeSeg& ls = p.ls;
    ls.seg = 0;
    ls.tile_begin = 0;
    ls.tile_end = (int32_t)nt;
    ls.sampled = plan_sample(d, k, &ls, &per_tile) ? 1 : 0;
    pl.n_large = 1;
    pl.n_tiles = (int)nt;
    pl.slot = kSlotMin;
    if (ls.sampled) {
      pl.slot = plan_slots(per_tile);
      if (nt * (int64_t)pl.slot > kStaticMaxSlots) return LAGS_ECAPACITY;  // a dense layer needs more slots than the array has
      const int64_t nwc = (nt + kWaveTiles - 1) / kWaveTiles;
      ls.chunk_begin = 0;
      ls.chunk_end = (int32_t)nt;
      ls.wchunk_begin = 0;
      ls.fused = nt <= kFusedTiles ? 1 : 0;
      pl.n_sampled = 1;
      pl.n_chunks = (int)nt;
      pl.n_wchunks = (int)((nwc + 3) / 4 * 4);
      if (!ls.fused) {
        ls.group_begin = 0;
        ls.group_end = (int32_t)((nwc + kGroupWaves - 1) / kGroupWaves);
        ls.group_h_begin = 0;
        ls.group_h_end = (int32_t)((nt + kCountTiles - 1) / kCountTiles);
        pl.n_groups = ls.group_end;
        pl.n_hparts = ls.group_h_end;
        pl.n_multi = 1;
      }
    } else {
      pl.has_dense = true;
    }
    pl.n_finish_small = finish_small(ls) ? 1 : 0;
    p.n_tiles = pl.n_tiles;
    p.n_groups = pl.n_groups;
    p.n_hparts = pl.n_hparts;
  }
  DeviceGuard g(device);
  if (!g.ok) return LAGS_EHIP;
  unsigned char* base = nullptr;
  const int rc = device_scratch(device, &base);
  if (rc != LAGS_OK) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  {
    const int n = p.n_tiles > 1 ? p.n_tiles : 1;
    hipLaunchKernelGGL(k_plan_layer, dim3((n + 255) / 256), dim3(256), 0, s, base, p);
    if (hipGetLastError() != hipSuccess) return LAGS_EHIP;
  }
  const SegDesc* segs = reinterpret_cast<const SegDesc*>(base + kLayout.segs);
  if (cls < kSmallClasses) {
    if (launch_small(cls, 1, segs, reinterpret_cast<const int32_t*>(base + kLayout.list), grad, residual, lr, out_idx,
                     out_val, s, nullptr) != hipSuccess)
      return LAGS_EHIP;
    return LAGS_OK;
  }
  pl.lsegs = reinterpret_cast<const LargeSeg*>(base + kLayout.lseg);
  pl.tiles = reinterpret_cast<const TileDesc*>(base + kLayout.tiles);
  pl.groups = reinterpret_cast<const GroupDesc*>(base + kLayout.groups);
  pl.hparts = reinterpret_cast<const GroupDesc*>(base + kLayout.hparts);
  pl.multi = reinterpret_cast<const int32_t*>(base + kLayout.multi);
  pl.fin_small = pl.multi;  // the one large layer, index 0, is in one of the two lists
  pl.fin_other = pl.multi;
  Scratch sc;
  sc.lstate = reinterpret_cast<LState*>(base + kLayout.lstate);
  sc.chunk_cnt = reinterpret_cast<uint32_t*>(base + kLayout.chunk_cnt);
  sc.slots = reinterpret_cast<uint2*>(base + kLayout.slots);
  sc.wgt = reinterpret_cast<uint32_t*>(base + kLayout.wgt);
  sc.band = reinterpret_cast<uint2*>(base + kLayout.band);
  sc.band_cnt = reinterpret_cast<uint32_t*>(base + kLayout.band_cnt);
  sc.bh_part = reinterpret_cast<uint32_t*>(base + kLayout.bh_part);
  sc.coarse_part = reinterpret_cast<uint32_t*>(base + kLayout.coarse_part);
  sc.part_info = reinterpret_cast<uint4*>(base + kLayout.part_info);
  sc.ghist = reinterpret_cast<uint32_t*>(base + kLayout.ghist);
  sc.dstate = reinterpret_cast<DState*>(base + kLayout.dstate);
  sc.tile_gt = reinterpret_cast<uint32_t*>(base + kLayout.tile_gt);
  sc.tile_eq = reinterpret_cast<uint32_t*>(base + kLayout.tile_eq);
  sc.items = reinterpret_cast<int32_t*>(base + kLayout.items);
  sc.fail_flag = reinterpret_cast<uint32_t*>(base + kLayout.fail);   // nobody reads it: a rejected guess is
                                                                      // always served inside the same launches
  if (launch_large_prep(pl, sc, segs, grad, residual, lr, /*chain=*/false, s, nullptr) != hipSuccess) return LAGS_EHIP;
  if (launch_large(pl, sc, segs, grad, residual, lr, out_idx, out_val, /*chain=*/false, s, nullptr) != hipSuccess)
    return LAGS_EHIP;
  return LAGS_OK;
}

}  // extern "C"
