// Host side of liblags.so: the C ABI declared in include/lags.h.
// Validates arguments, prepares layer tables (k per layer, output positions, size
// classes, tile lists), owns the scratch arena and enqueues the kernels.
#include "../../include/lags.h"
#include "lags_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <map>
#include <new>
#include <utility>
#include <vector>

using namespace lags;

// A device buffer that only ever grows.  The larger buffer is allocated before the old one is
// given up, so a failed allocation leaves the buffer (and every table that uses it) intact.
// `retired`: if not null the old allocation is kept there instead of being freed (a captured
// HIP graph may still hold its address).
struct DevBuf {
  void* p = nullptr;
  size_t bytes = 0;
  int grow(size_t need, std::vector<void*>* retired) {
    if (need <= bytes) return LAGS_OK;
    void* q = nullptr;
    if (hipMalloc(&q, need) != hipSuccess) return LAGS_ENOMEM;
    if (p) {
      bool kept = false;
      if (retired) {
        try {
          retired->push_back(p);
          kept = true;
        } catch (const std::bad_alloc&) {
        }
        if (!kept) {  // cannot keep the old buffer alive: refuse to move it
          (void)hipFree(q);
          return LAGS_ENOMEM;
        }
      } else {
        (void)hipFree(p);
      }
    }
    p = q;
    bytes = need;
    return LAGS_OK;
  }
  void release() {
    if (p) (void)hipFree(p);
    p = nullptr;
    bytes = 0;
  }
};

struct lags_ctx {
  int device = 0;
  // scratch of the large layers' path, sized for the largest table created so far
  DevBuf bh_part, coarse_part, part_info, lstate, chunk_cnt, slots, wgt, band, band_cnt, ghist, dstate, tile_gt, tile_eq, items;
  DevBuf bounds;   // merge: P rows of tile start positions, sized at the first merge call that needs it
  DevBuf partials; // delta metric: two doubles per merge tile
  // Once a call of this context has been recorded by stream capture, scratch that has to grow is
  // not freed but kept until lags_destroy: the recorded graph holds its address.
  bool captured = false;
  std::vector<void*> retired;
  // A pinned host word that a kernel sets when a sampled layer's guess is rejected.  The next
  // calls then also enqueue the multi-pass kernels, so that rejected layers are selected by many
  // workgroups instead of one (results are the same either way).
  uint32_t* fail_host = nullptr;
  uint32_t* fail_dev = nullptr;
  int armed_calls = 0;   // calls left that enqueue the multi-pass kernels
  int chain_mode = 0;    // 0: as above; 1: always enqueue them; 2: never (diagnostic setting)
  std::map<std::pair<int64_t, int64_t>, lags_table*> layer_tables;  // (d, k) -> one-layer table
  Prof prof;
  // side stream (default priority) on which the small layers' kernels run beside the large
  // layers' pipeline; forked from and joined to the caller's stream with events in every call
  hipStream_t aux = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr, ev_side = nullptr;
  std::vector<void*>* retire_list() { return captured ? &retired : nullptr; }
  Scratch scratch() const {
    Scratch sc;
    sc.bh_part = static_cast<uint32_t*>(bh_part.p);
    sc.coarse_part = static_cast<uint32_t*>(coarse_part.p);
    sc.part_info = static_cast<uint4*>(part_info.p);
    sc.lstate = static_cast<LState*>(lstate.p);
    sc.chunk_cnt = static_cast<uint32_t*>(chunk_cnt.p);
    sc.slots = static_cast<uint2*>(slots.p);
    sc.wgt = static_cast<uint32_t*>(wgt.p);
    sc.band = static_cast<uint2*>(band.p);
    sc.band_cnt = static_cast<uint32_t*>(band_cnt.p);
    sc.ghist = static_cast<uint32_t*>(ghist.p);
    sc.dstate = static_cast<DState*>(dstate.p);
    sc.tile_gt = static_cast<uint32_t*>(tile_gt.p);
    sc.tile_eq = static_cast<uint32_t*>(tile_eq.p);
    sc.items = static_cast<int32_t*>(items.p);
    sc.fail_flag = fail_dev;
    return sc;
  }
};

struct lags_table {
  lags_ctx* ctx = nullptr;
  int32_t n = 0;
  int64_t total_k = 0;
  int64_t span_lo = 0, span_hi = 0;            // [min offset, max offset + d)
  std::vector<SegDesc> segs;                   // host copy
  std::vector<LargeSeg> lsegs;                 // host copy
  int n_small[kSmallClasses] = {0, 0};
  MergePlan mplan;
  LargePlan plan;                              // device pointers below, owned by the table
  SegDesc* d_segs = nullptr;
  int32_t* d_small[kSmallClasses] = {nullptr, nullptr};
  LargeSeg* d_lsegs = nullptr;
  TileDesc* d_tiles = nullptr;
  GroupDesc* d_groups = nullptr;
  GroupDesc* d_hparts = nullptr;
  int32_t* d_multi = nullptr;
  int32_t* d_fin_small = nullptr;
  int32_t* d_fin_other = nullptr;
  MTile* d_mtiles = nullptr;
  BChunk* d_bchunks = nullptr;
  int32_t* d_seg_mtile0 = nullptr;
};

namespace lags {

// Plan of the threshold guess for a large layer of d elements keeping k: how many sample
// pieces and which ranks of the sample become the threshold and the estimate of the k-th
// largest key.  Returns false if the layer is not worth sampling (k too large for the slots).
bool plan_sample(int64_t d, int64_t k, LargeSeg* ls, double* per_tile) {
  int64_t pieces, stride;
  const int64_t piece_len = kSamplePiece;
  const int64_t max_pieces = d <= kSampleSmallElems ? kSamplePiecesSmall : kSamplePieces;
  if (d >= max_pieces * piece_len) {
    pieces = max_pieces;
    stride = d / max_pieces;
  } else {
    pieces = (d + piece_len - 1) / piece_len;
    stride = piece_len;
  }
  const double m = (double)std::min<int64_t>(d, pieces * piece_len);
  const double fk = (double)k * m / (double)d;
  // the sample's rank-j key admits about j/m of the layer; j is fk plus five standard
  // deviations of the sampled count plus a constant: fewer than k candidates (which costs the
  // slow selection of that layer in that call) then has a probability below 1e-6
  const double jd = std::ceil(fk + 5.0 * std::sqrt(fk) + 8.0);
  if (jd > m) return false;
  // expected candidates per tile must stay well inside the largest slot size
  *per_tile = jd / m * (double)kTile;
  if (*per_tile > (double)kSlotMax * 0.5) return false;
  // The candidates between the threshold and the expected k-th largest key, (jd - fk) / fk * k of
  // them, spread over at least 512 buckets; the bucket of the k-th largest key must hold no more
  // than kBandCap entries (kBandCapSmall where a small workgroup finishes the layer).  Layers
  // that keep so many entries that this leaves less than a factor 4 take the multi-pass route.
  const int64_t band_cap = (d + kTile - 1) / kTile <= kFinishSmallTiles ? kBandCapSmall : kBandCap;
  if ((jd - fk) / fk * (double)k / 512.0 > (double)band_cap / 4.0) return false;
  ls->sample_rank = (int32_t)jd;
  // the sample's best estimate of the k-th largest key: it sets the width of the candidate buckets
  ls->sample_rank_hi = (int32_t)std::max(1.0, std::floor(fk));
  ls->sample_pieces = (int32_t)pieces;
  ls->sample_stride = (int32_t)stride;
  return true;
}

int plan_slots(double max_per_tile) {
  int slot = kSlotMin;
  while ((double)slot < 8.0 * max_per_tile && slot < kSlotMax) slot *= 2;
  return slot;
}

}  // namespace lags

namespace {

constexpr size_t kMaxLayerPlans = 4096;  // cached one-layer plans of lags_sparsify_layer

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

template <typename T>
int upload(T** dst, const std::vector<T>& src) {
  *dst = nullptr;
  if (src.empty()) return LAGS_OK;
  if (hipMalloc(reinterpret_cast<void**>(dst), src.size() * sizeof(T)) != hipSuccess) {
    *dst = nullptr;
    return LAGS_ENOMEM;
  }
  if (hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return LAGS_EHIP;
  return LAGS_OK;
}

bool ranges_overlap(const void* a, int64_t abytes, const void* b, int64_t bbytes) {
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a0 < b0 + (uintptr_t)bbytes && b0 < a0 + (uintptr_t)abytes;
}

std::vector<DevBuf*> all_bufs(lags_ctx* ctx) {
  return {&ctx->bh_part, &ctx->coarse_part, &ctx->part_info, &ctx->lstate, &ctx->chunk_cnt, &ctx->slots, &ctx->wgt, &ctx->band, &ctx->band_cnt, &ctx->ghist,
          &ctx->dstate, &ctx->tile_gt, &ctx->tile_eq, &ctx->items, &ctx->bounds, &ctx->partials};
}

void free_table_device(lags_table* t) {
  if (t->d_segs) (void)hipFree(t->d_segs);
  for (int c = 0; c < kSmallClasses; ++c)
    if (t->d_small[c]) (void)hipFree(t->d_small[c]);
  if (t->d_lsegs) (void)hipFree(t->d_lsegs);
  if (t->d_tiles) (void)hipFree(t->d_tiles);
  if (t->d_groups) (void)hipFree(t->d_groups);
  if (t->d_hparts) (void)hipFree(t->d_hparts);
  if (t->d_multi) (void)hipFree(t->d_multi);
  if (t->d_fin_small) (void)hipFree(t->d_fin_small);
  if (t->d_fin_other) (void)hipFree(t->d_fin_other);
  if (t->d_mtiles) (void)hipFree(t->d_mtiles);
  if (t->d_bchunks) (void)hipFree(t->d_bchunks);
  if (t->d_seg_mtile0) (void)hipFree(t->d_seg_mtile0);
}

// Build a table from explicit (offset, d, k) triples.
int build_table(lags_ctx* ctx, const std::vector<int64_t>& off, const std::vector<int64_t>& d,
                const std::vector<int64_t>& k, lags_table** out) {
  const int32_t n = (int32_t)off.size();
  lags_table* t = new (std::nothrow) lags_table();
  if (!t) return LAGS_ENOMEM;
  t->ctx = ctx;
  t->n = n;
  std::vector<int32_t> small[kSmallClasses], multi;
  std::vector<TileDesc> tiles;
  std::vector<MTile> mtiles;
  std::vector<GroupDesc> groups, hparts;
  std::vector<BChunk> bchunks;
  std::vector<int32_t> seg_mtile0;
  int64_t n_chunks = 0;        // tiles of sampled layers: each owns `slot` candidate slots
  int64_t n_wchunks = 0;       // runs of kWaveTiles such tiles
  double max_per_tile = 0.0;   // largest expected candidate count per tile over the sampled layers
  constexpr int64_t kMaxTiles = 1 << 28;
  int fuse_limit = kFusedTiles;
  for (int32_t l = 0; l < n; ++l) {
    LargeSeg probe = {};
    double unused = 0.0;
    if (d[l] > (int64_t)kFusedTiles * kTile && plan_sample(d[l], k[l], &probe, &unused)) fuse_limit = kFusedTilesShared;
  }
  try {
    t->segs.resize(n);
    int64_t outpos = 0;
    t->span_lo = off[0];
    t->span_hi = off[0] + d[0];
    for (int32_t l = 0; l < n; ++l) {
      SegDesc& s = t->segs[l];
      s.offset = off[l];
      s.out_offset = outpos;
      s.d = (int32_t)d[l];
      s.k = (int32_t)k[l];
      outpos += k[l];
      t->span_lo = std::min(t->span_lo, off[l]);
      t->span_hi = std::max(t->span_hi, off[l] + d[l]);
      if (d[l] <= kSmall0) small[0].push_back(l);
      else if (d[l] <= kSmall1) small[1].push_back(l);
      else {
        LargeSeg ls = {};
        const int32_t li = (int32_t)t->lsegs.size();
        ls.seg = l;
        double per_tile = 0.0;
        ls.sampled = plan_sample(d[l], k[l], &ls, &per_tile) ? 1 : 0;
        ls.tile_begin = (int32_t)tiles.size();
        const int64_t nt = (d[l] + kTile - 1) / kTile;
        if ((int64_t)tiles.size() + nt > kMaxTiles) { delete t; return LAGS_ECAPACITY; }
        if (ls.sampled) {
          max_per_tile = std::max(max_per_tile, per_tile);
          ls.chunk_begin = (int32_t)n_chunks;
          ls.chunk_end = (int32_t)(n_chunks + nt);
          ls.wchunk_begin = (int32_t)n_wchunks;   // a multiple of 4: k_group_p moves four entries at a time
          const int64_t nwc = (nt + kWaveTiles - 1) / kWaveTiles;
          n_wchunks += (nwc + 3) / 4 * 4;
          ls.fused = nt <= fuse_limit ? 1 : 0;
          if (!ls.fused) {
            ls.group_begin = (int32_t)groups.size();
            const int64_t ng = (nwc + kGroupWaves - 1) / kGroupWaves;
            for (int64_t g = 0; g < ng; ++g) {
              GroupDesc gd;
              gd.lseg = li;
              gd.first = (int32_t)g;
              groups.push_back(gd);
            }
            ls.group_end = (int32_t)groups.size();
            ls.group_h_begin = (int32_t)hparts.size();
            for (int64_t h = 0; h * kCountTiles < nt; ++h) {
              GroupDesc hp;
              hp.lseg = li;
              hp.first = (int32_t)h;
              hparts.push_back(hp);
            }
            ls.group_h_end = (int32_t)hparts.size();
            multi.push_back(li);
          }
        } else {
          t->plan.has_dense = true;
        }
        for (int64_t i = 0; i < nt; ++i) {
          TileDesc td;
          td.start = off[l] + i * kTile;
          td.n = (int32_t)std::min<int64_t>(kTile, d[l] - i * kTile);
          td.seg = li;
          td.local0 = (int32_t)(i * kTile);
          td.ctile = ls.sampled ? (int32_t)(n_chunks + i) : -1;
          tiles.push_back(td);
        }
        if (ls.sampled) n_chunks += nt;
        ls.tile_end = (int32_t)tiles.size();
        t->lsegs.push_back(ls);
      }
      const int64_t nmt = (d[l] + kMergeTile - 1) / kMergeTile;
      if ((int64_t)mtiles.size() + nmt > kMaxTiles) { delete t; return LAGS_ECAPACITY; }
      seg_mtile0.push_back((int32_t)mtiles.size());
      for (int64_t j0 = 0; j0 < k[l]; j0 += kBoundChunk) {
        BChunk bc;
        bc.seg = l;
        bc.j0 = (int32_t)j0;
        bc.slot0 = (int32_t)mtiles.size() + l;   // every earlier layer owns one extra (end) slot
        bc.ntiles = (int32_t)nmt;
        bchunks.push_back(bc);
      }
      for (int64_t i = 0; i < nmt; ++i) {
        MTile mt;
        mt.start = off[l] + i * kMergeTile;
        mt.out_offset = s.out_offset;
        mt.n = (int32_t)std::min<int64_t>(kMergeTile, d[l] - i * kMergeTile);
        mt.seg = l;
        mt.local0 = (int32_t)(i * kMergeTile);
        mt.k = (int32_t)k[l];
        mtiles.push_back(mt);
      }
    }
    t->total_k = outpos;
    seg_mtile0.push_back((int32_t)mtiles.size());
  } catch (const std::bad_alloc&) {
    delete t;
    return LAGS_ENOMEM;
  }
  for (int c = 0; c < kSmallClasses; ++c) t->n_small[c] = (int)small[c].size();
  t->mplan.n_layers = n;
  t->mplan.n_mtiles = (int)mtiles.size();
  t->mplan.n_bchunks = (int)bchunks.size();
  t->mplan.nb = (int)mtiles.size() + n;
  LargePlan& pl = t->plan;
  pl.n_large = (int)t->lsegs.size();
  pl.n_tiles = (int)tiles.size();
  pl.n_chunks = (int)n_chunks;
  pl.n_wchunks = (int)n_wchunks;
  pl.n_groups = (int)groups.size();
  pl.n_multi = (int)multi.size();
  pl.n_hparts = (int)hparts.size();
  std::vector<int32_t> fin_small, fin_other;
  for (size_t li = 0; li < t->lsegs.size(); ++li) {
    const LargeSeg& ls = t->lsegs[li];
    pl.n_sampled += ls.sampled;
    (finish_small(ls) ? fin_small : fin_other).push_back((int32_t)li);
  }
  pl.n_finish_small = (int)fin_small.size();
  // candidates cluster (e.g. the few non-zero rows of an embedding gradient), so a tile may
  // hold several times the layer's average: the slots leave a factor 8 where they can
  pl.slot = plan_slots(max_per_tile);

  int rc = upload(&t->d_segs, t->segs);
  for (int c = 0; c < kSmallClasses && rc == LAGS_OK; ++c) rc = upload(&t->d_small[c], small[c]);
  if (rc == LAGS_OK) rc = upload(&t->d_lsegs, t->lsegs);
  if (rc == LAGS_OK) rc = upload(&t->d_tiles, tiles);
  if (rc == LAGS_OK) rc = upload(&t->d_groups, groups);
  if (rc == LAGS_OK) rc = upload(&t->d_hparts, hparts);
  if (rc == LAGS_OK) rc = upload(&t->d_multi, multi);
  if (rc == LAGS_OK) rc = upload(&t->d_fin_small, fin_small);
  if (rc == LAGS_OK) rc = upload(&t->d_fin_other, fin_other);
  if (rc == LAGS_OK) rc = upload(&t->d_mtiles, mtiles);
  if (rc == LAGS_OK) rc = upload(&t->d_bchunks, bchunks);
  if (rc == LAGS_OK) rc = upload(&t->d_seg_mtile0, seg_mtile0);
  t->mplan.mtiles = t->d_mtiles;
  t->mplan.bchunks = t->d_bchunks;
  t->mplan.seg_mtile0 = t->d_seg_mtile0;
  pl.lsegs = t->d_lsegs;
  pl.tiles = t->d_tiles;
  pl.groups = t->d_groups;
  pl.hparts = t->d_hparts;
  pl.multi = t->d_multi;
  pl.fin_small = t->d_fin_small;
  pl.fin_other = t->d_fin_other;
  if (pl.n_large > 0) {
    std::vector<void*>* rl = ctx->retire_list();
    const size_t nl = (size_t)pl.n_large;
    if (rc == LAGS_OK) rc = ctx->bh_part.grow((size_t)pl.n_hparts * kFineBins * sizeof(uint32_t), rl);
    if (rc == LAGS_OK) rc = ctx->coarse_part.grow((size_t)pl.n_hparts * kCoarseBins * sizeof(uint32_t), rl);
    if (rc == LAGS_OK) rc = ctx->part_info.grow((size_t)pl.n_hparts * sizeof(uint4), rl);
    if (rc == LAGS_OK) rc = ctx->lstate.grow(nl * sizeof(LState), rl);
    if (rc == LAGS_OK) rc = ctx->chunk_cnt.grow((size_t)pl.n_chunks * sizeof(uint32_t), rl);
    if (rc == LAGS_OK) rc = ctx->slots.grow((size_t)pl.n_chunks * (size_t)pl.slot * sizeof(uint2), rl);
    if (rc == LAGS_OK) rc = ctx->wgt.grow((size_t)pl.n_wchunks * sizeof(uint32_t), rl);
    if (rc == LAGS_OK) rc = ctx->band.grow((size_t)pl.n_groups * kGroupBand * sizeof(uint2), rl);
    if (rc == LAGS_OK) rc = ctx->band_cnt.grow((size_t)pl.n_groups * sizeof(uint32_t), rl);
    if (rc == LAGS_OK) rc = ctx->ghist.grow((nl * kHistStride + 16) * sizeof(uint32_t), rl);
    if (rc == LAGS_OK) rc = ctx->dstate.grow(nl * sizeof(DState), rl);
    if (rc == LAGS_OK) rc = ctx->tile_gt.grow((size_t)pl.n_tiles * sizeof(uint32_t), rl);
    if (rc == LAGS_OK) rc = ctx->tile_eq.grow((size_t)pl.n_tiles * sizeof(uint32_t), rl);
    if (rc == LAGS_OK) rc = ctx->items.grow((size_t)pl.n_tiles * sizeof(int32_t), rl);
  }
  if (rc != LAGS_OK) {
    free_table_device(t);
    delete t;
    return rc;
  }
  *out = t;
  return LAGS_OK;
}

int run_sparsify(lags_ctx* ctx, const lags_table* t, const float* grad, float* res, float lr,
                 int32_t* out_idx, float* out_val, hipStream_t s) {
  // a call that is being recorded into a graph pins the scratch it uses (see DevBuf::grow)
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone) ctx->captured = true;
  // Do the multi-pass kernels run in this call?  Always for tables with layers that are not
  // sampled; otherwise for a number of calls after a kernel reported a rejected guess.
  bool chain = t->plan.has_dense;
  if (t->plan.n_large > 0) {
    if (ctx->fail_host && *static_cast<volatile uint32_t*>(ctx->fail_host)) {
      *static_cast<volatile uint32_t*>(ctx->fail_host) = 0u;
      ctx->armed_calls = 64;
    }
    if (ctx->armed_calls > 0) {
      chain = true;
      --ctx->armed_calls;
    }
    if (ctx->chain_mode == 1) chain = true;
    if (ctx->chain_mode == 2) chain = t->plan.has_dense;
  }
  ProfScope whole(&ctx->prof, K_SPARSIFY_CALL, s);
  // Small and large layers touch disjoint parts of every buffer, so the small layers' kernels
  // run on the side stream while the large layers' pipeline occupies the caller's stream.  The
  // side stream starts after the threshold guesses: those are short and everything else waits
  // for them, and the small layers' workgroups would otherwise take their wave slots.
  int rc = LAGS_OK;
  if (launch_large_prep(t->plan, ctx->scratch(), t->d_segs, grad, res, lr, chain, s, &ctx->prof) != hipSuccess)
    rc = LAGS_EHIP;
  const bool have_small = t->n_small[0] + t->n_small[1] > 0;
  bool fork = rc == LAGS_OK && ctx->aux && have_small && t->plan.n_large > 0;
  if (fork && (hipEventRecord(ctx->ev_fork, s) != hipSuccess ||
               hipStreamWaitEvent(ctx->aux, ctx->ev_fork, 0) != hipSuccess))
    fork = false;
  hipStream_t ss = fork ? ctx->aux : s;
  for (int c = 0; c < kSmallClasses && rc == LAGS_OK; ++c) {
    if (launch_small(c, t->n_small[c], t->d_segs, t->d_small[c], grad, res, lr, out_idx, out_val, ss, &ctx->prof) != hipSuccess)
      rc = LAGS_EHIP;
  }
  // the layers that one small workgroup finishes need nothing from the kernels of the layers
  // finished by groups: when the table has both, the side stream takes them after the streaming pass
  const LargePlan& pl = t->plan;
  const bool offload = rc == LAGS_OK && ctx->aux && !chain && pl.n_finish_small > 0 && pl.n_finish_small < pl.n_large;
  if (rc == LAGS_OK &&
      launch_large(pl, ctx->scratch(), t->d_segs, grad, res, lr, out_idx, out_val, chain, s, &ctx->prof,
                   offload ? ctx->aux : nullptr, ctx->ev_side) != hipSuccess)
    rc = LAGS_EHIP;
  // always join what was forked, also on an error path, so the caller's stream stays ordered
  if (fork || offload) {
    if (hipEventRecord(ctx->ev_join, ctx->aux) != hipSuccess || hipStreamWaitEvent(s, ctx->ev_join, 0) != hipSuccess)
      rc = LAGS_EHIP;
  }
  return rc;
}

}  // namespace

extern "C" {

int64_t lags_topk_count(int64_t d, double rho) {
  if (d < 1 || !(rho > 0.0) || !(rho <= 1.0)) return -1;
  int64_t k = (int64_t)std::ceil(rho * (double)d);
  if (k < 1) k = 1;
  if (k > d) k = d;
  return k;
}

int lags_create(lags_ctx** out, int device) {
  if (!out) return LAGS_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess) return LAGS_EHIP;
  if (device < 0 || device >= count) return LAGS_EINVAL;
  lags_ctx* c = new (std::nothrow) lags_ctx();
  if (!c) return LAGS_ENOMEM;
  c->device = device;
  {
    DeviceGuard g(device);
    // LAGS_SIDE_STREAM=0 keeps every kernel on the caller's stream (for tools that serialise
    // the dispatches of all queues, such as counter collection)
    const char* side = std::getenv("LAGS_SIDE_STREAM");
    const bool want_side = !(side && side[0] == '0' && side[1] == '\0');
    if (g.ok && want_side && hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking) == hipSuccess) {
      if (hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
          hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess ||
          hipEventCreateWithFlags(&c->ev_side, hipEventDisableTiming) != hipSuccess) {
        if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
        if (c->ev_join) (void)hipEventDestroy(c->ev_join);
        if (c->ev_side) (void)hipEventDestroy(c->ev_side);
        (void)hipStreamDestroy(c->aux);
        c->aux = nullptr;   // everything then runs on the caller's stream
        c->ev_fork = c->ev_join = c->ev_side = nullptr;
      }
    } else {
      c->aux = nullptr;
    }
    // the word through which kernels report a rejected guess: pinned, mapped host memory
    void* hp = nullptr;
    void* dp = nullptr;
    if (!g.ok || hipHostMalloc(&hp, sizeof(uint32_t), hipHostMallocMapped) != hipSuccess ||
        hipHostGetDevicePointer(&dp, hp, 0) != hipSuccess) {
      if (hp) (void)hipHostFree(hp);
      if (c->aux) {
        (void)hipStreamDestroy(c->aux);
        (void)hipEventDestroy(c->ev_fork);
        (void)hipEventDestroy(c->ev_join);
        (void)hipEventDestroy(c->ev_side);
      }
      delete c;
      return g.ok ? LAGS_ENOMEM : LAGS_EHIP;
    }
    c->fail_host = static_cast<uint32_t*>(hp);
    c->fail_dev = static_cast<uint32_t*>(dp);
    *c->fail_host = 0u;
  }
  *out = c;
  return LAGS_OK;
}

int lags_destroy(lags_ctx* ctx) {
  if (!ctx) return LAGS_EINVAL;
  DeviceGuard g(ctx->device);
  (void)lags_profile_reset(ctx);
  if (ctx->aux) {
    (void)hipStreamSynchronize(ctx->aux);
    (void)hipStreamDestroy(ctx->aux);
    (void)hipEventDestroy(ctx->ev_fork);
    (void)hipEventDestroy(ctx->ev_join);
    (void)hipEventDestroy(ctx->ev_side);
  }
  for (auto& kv : ctx->layer_tables) {
    free_table_device(kv.second);
    delete kv.second;
  }
  (void)hipDeviceSynchronize();  // no kernel may still write the pinned word or the scratch
  for (DevBuf* b : all_bufs(ctx)) b->release();
  for (void* p : ctx->retired) (void)hipFree(p);
  if (ctx->fail_host) (void)hipHostFree(ctx->fail_host);
  delete ctx;
  return LAGS_OK;
}

int lags_table_create(lags_ctx* ctx, const lags_layer_desc* layers, int32_t n, lags_table** out) {
  if (!ctx || !layers || !out || n < 1) return LAGS_EINVAL;
  *out = nullptr;
  std::vector<int64_t> off, d, k;
  std::vector<std::pair<int64_t, int64_t>> order;
  try {
    off.resize(n); d.resize(n); k.resize(n); order.resize(n);
  } catch (const std::bad_alloc&) {
    return LAGS_ENOMEM;
  }
  for (int32_t l = 0; l < n; ++l) {
    if (layers[l].offset < 0 || layers[l].d < 1 || layers[l].d > 0x7FFFFFFFLL) return LAGS_EINVAL;
    if (layers[l].offset > (int64_t)1 << 60) return LAGS_EINVAL;
    const int64_t kk = lags_topk_count(layers[l].d, layers[l].rho);
    if (kk < 1) return LAGS_EINVAL;
    off[l] = layers[l].offset;
    d[l] = layers[l].d;
    k[l] = kk;
    order[l] = std::make_pair(off[l], d[l]);
  }
  std::sort(order.begin(), order.end());
  for (int32_t l = 1; l < n; ++l)
    if (order[l - 1].first + order[l - 1].second > order[l].first) return LAGS_EINVAL;  // layers overlap
  DeviceGuard g(ctx->device);
  if (!g.ok) return LAGS_EHIP;
  return build_table(ctx, off, d, k, out);
}

int lags_table_destroy(lags_table* t) {
  if (!t) return LAGS_EINVAL;
  DeviceGuard g(t->ctx->device);
  free_table_device(t);
  delete t;
  return LAGS_OK;
}

int32_t lags_table_num_layers(const lags_table* t) { return t ? t->n : -1; }
int64_t lags_table_total_k(const lags_table* t) { return t ? t->total_k : -1; }
int64_t lags_table_k(const lags_table* t, int32_t l) { return (t && l >= 0 && l < t->n) ? t->segs[l].k : -1; }
int64_t lags_table_out_offset(const lags_table* t, int32_t l) {
  return (t && l >= 0 && l < t->n) ? t->segs[l].out_offset : -1;
}

int lags_sparsify_layer(lags_ctx* ctx, const float* grad, float* residual, int64_t d, float lr, int64_t k,
                        int32_t* out_idx, float* out_val, void* hip_stream) {
  if (!ctx || !grad || !residual || !out_idx || !out_val) return LAGS_EINVAL;
  if (d < 1 || d > 0x7FFFFFFFLL || k < 1 || k > d || !std::isfinite(lr)) return LAGS_EINVAL;
  const int64_t db = d * 4, kb = k * 4;
  if (ranges_overlap(grad, db, residual, db) || ranges_overlap(out_idx, kb, out_val, kb) ||
      ranges_overlap(grad, db, out_idx, kb) || ranges_overlap(grad, db, out_val, kb) ||
      ranges_overlap(residual, db, out_idx, kb) || ranges_overlap(residual, db, out_val, kb))
    return LAGS_EINVAL;
  DeviceGuard g(ctx->device);
  if (!g.ok) return LAGS_EHIP;
  lags_table* t = nullptr;
  auto it = ctx->layer_tables.find(std::make_pair(d, k));
  if (it != ctx->layer_tables.end()) {
    t = it->second;
  } else {
    // the cache of one-layer plans is bounded: when full it is emptied (hipFree waits for the
    // device, so no launch still reads the plans that go away)
    if (ctx->layer_tables.size() >= kMaxLayerPlans) {
      for (auto& kv : ctx->layer_tables) {
        free_table_device(kv.second);
        delete kv.second;
      }
      ctx->layer_tables.clear();
    }
    std::vector<int64_t> off(1, 0), dd(1, d), kk(1, k);
    int rc = build_table(ctx, off, dd, kk, &t);
    if (rc != LAGS_OK) return rc;
    try {
      ctx->layer_tables[std::make_pair(d, k)] = t;
    } catch (const std::bad_alloc&) {
      free_table_device(t);
      delete t;
      return LAGS_ENOMEM;
    }
  }
  return run_sparsify(ctx, t, grad, residual, lr, out_idx, out_val, (hipStream_t)hip_stream);
}

int lags_sparsify_model(lags_ctx* ctx, const lags_table* t, const float* grad_flat, float* residual_flat,
                        float lr, int32_t* out_idx, float* out_val, void* hip_stream) {
  if (!ctx || !t || t->ctx != ctx || !grad_flat || !residual_flat || !out_idx || !out_val) return LAGS_EINVAL;
  if (!std::isfinite(lr)) return LAGS_EINVAL;
  const int64_t lo = t->span_lo * 4, db = (t->span_hi - t->span_lo) * 4, kb = t->total_k * 4;
  const char* gp = reinterpret_cast<const char*>(grad_flat) + lo;
  const char* rp = reinterpret_cast<const char*>(residual_flat) + lo;
  if (ranges_overlap(gp, db, rp, db) || ranges_overlap(out_idx, kb, out_val, kb) ||
      ranges_overlap(gp, db, out_idx, kb) || ranges_overlap(gp, db, out_val, kb) ||
      ranges_overlap(rp, db, out_idx, kb) || ranges_overlap(rp, db, out_val, kb))
    return LAGS_EINVAL;
  DeviceGuard g(ctx->device);
  if (!g.ok) return LAGS_EHIP;
  return run_sparsify(ctx, t, grad_flat, residual_flat, lr, out_idx, out_val, (hipStream_t)hip_stream);
}

namespace {
// Validation and launch shared by the three merge-type entry points.
int run_merge(int mode, lags_ctx* ctx, const lags_table* t, const int32_t* idx, const float* val, int32_t P,
              int64_t stride_k, float* out, const float* res, int64_t res_stride, double* out3, void* hip_stream) {
  if (!ctx || !t || t->ctx != ctx || !idx || !val) return LAGS_EINVAL;
  if (P < 1 || P > kMaxWorkers || stride_k < t->total_k) return LAGS_EINVAL;
  const int64_t pb = ((int64_t)(P - 1) * stride_k + t->total_k) * 4;
  const int64_t lo = t->span_lo * 4, span = (t->span_hi - t->span_lo) * 4;
  if (mode == MERGE_DELTA) {
    if (!res || !out3 || res_stride < t->span_hi - t->span_lo) return LAGS_EINVAL;
    const int64_t ob = (int64_t)t->n * 3 * 8;
    const char* rp = reinterpret_cast<const char*>(res) + lo;
    const int64_t rb = (int64_t)(P - 1) * res_stride * 4 + span;
    if (ranges_overlap(out3, ob, idx, pb) || ranges_overlap(out3, ob, val, pb) || ranges_overlap(out3, ob, rp, rb))
      return LAGS_EINVAL;
  } else {
    if (!out) return LAGS_EINVAL;
    const char* up = reinterpret_cast<const char*>(out) + lo;
    if (ranges_overlap(up, span, idx, pb) || ranges_overlap(up, span, val, pb)) return LAGS_EINVAL;
  }
  DeviceGuard g(ctx->device);
  if (!g.ok) return LAGS_EHIP;
  // P rows of tile bounds (and the delta partial sums): these grow, with a synchronous
  // allocation, the first time a larger P or table is used
  {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing((hipStream_t)hip_stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone)
      ctx->captured = true;
  }
  if (ctx->bounds.grow((size_t)P * (size_t)t->mplan.nb * sizeof(int32_t), ctx->retire_list()) != LAGS_OK)
    return LAGS_ENOMEM;
  if (mode == MERGE_DELTA &&
      ctx->partials.grow((size_t)t->mplan.n_mtiles * 2 * sizeof(double), ctx->retire_list()) != LAGS_OK)
    return LAGS_ENOMEM;
  if (launch_merge(mode, t->mplan, static_cast<int32_t*>(ctx->bounds.p), t->d_segs, idx, val, P, stride_k, out, res,
                   res_stride, static_cast<double*>(ctx->partials.p), out3, (hipStream_t)hip_stream,
                   &ctx->prof) != hipSuccess)
    return LAGS_EHIP;
  return LAGS_OK;
}
}  // namespace

int lags_merge_sparse(lags_ctx* ctx, const lags_table* t, const int32_t* idx, const float* val, int32_t P,
                      int64_t stride_k, float* update_flat, void* hip_stream) {
  return run_merge(MERGE_UPDATE, ctx, t, idx, val, P, stride_k, update_flat, nullptr, 0, nullptr, hip_stream);
}

int lags_apply_sparse(lags_ctx* ctx, const lags_table* t, const int32_t* idx, const float* val, int32_t P,
                      int64_t stride_k, float* param_flat, void* hip_stream) {
  return run_merge(MERGE_APPLY, ctx, t, idx, val, P, stride_k, param_flat, nullptr, 0, nullptr, hip_stream);
}

int lags_delta_monitor(lags_ctx* ctx, const lags_table* t, const float* residual_flat, int64_t res_stride,
                       const int32_t* idx, const float* val, int32_t P, int64_t stride_k, double* out3,
                       void* hip_stream) {
  return run_merge(MERGE_DELTA, ctx, t, idx, val, P, stride_k, nullptr, residual_flat, res_stride, out3, hip_stream);
}

double lags_allgather_seconds(const lags_allgather_model* net, int64_t k) {
  if (!net || net->P < 1 || k < 0) return std::nan("");
  return ((double)(net->P - 1)) * (net->alpha + (8.0 * (double)k) * net->beta);
}

int lags_adaptive_ratios(const lags_allgather_model* net, const int64_t* d, const double* t_comp,
                         const double* t_spar, int32_t n, double c_u, int64_t* k_out, double* rho_out) {
  if (!net || !d || !t_comp || !t_spar || !k_out || n < 1) return LAGS_EINVAL;
  if (net->P < 1 || !(net->alpha >= 0.0) || !(net->beta >= 0.0) || !(c_u >= 1.0)) return LAGS_EINVAL;
  for (int32_t l = 0; l < n; ++l)
    if (d[l] < 1 || d[l] > 0x7FFFFFFFLL || !(t_comp[l] >= 0.0) || !(t_spar[l] >= 0.0)) return LAGS_EINVAL;
  for (int32_t l = 0; l < n; ++l) {
    const double budget = l == 0 ? 0.0 : t_comp[l - 1];
    // t_comm is non-decreasing in k (products and sums of non-negative doubles are monotone), so
    // the largest k that fits is found by bisection on the very predicate of Eq. 9
    auto fits = [&](int64_t k) { return lags_allgather_seconds(net, k) + t_spar[l] <= budget; };
    int64_t k_fit = 0;
    if (fits(1)) {
      if (fits(d[l])) {
        k_fit = d[l];
      } else {
        int64_t lo = 1, hi = d[l];   // fits(lo), !fits(hi)
        while (hi - lo > 1) {
          const int64_t mid = lo + (hi - lo) / 2;
          if (fits(mid)) lo = mid; else hi = mid;
        }
        k_fit = lo;
      }
    }
    int64_t k_min = (int64_t)std::ceil((double)d[l] / c_u);   // c = d/k <= c_u
    if (k_min < 1) k_min = 1;
    if (k_min > d[l]) k_min = d[l];
    const int64_t k = std::max(k_fit, k_min);
    k_out[l] = k;
    if (rho_out) {
      double rho = (double)k / (double)d[l];
      if (rho > 1.0) rho = 1.0;
      for (int guard = 0; guard < 64 && lags_topk_count(d[l], rho) > k; ++guard) rho = std::nextafter(rho, 0.0);
      for (int guard = 0; guard < 64 && lags_topk_count(d[l], rho) < k; ++guard) rho = std::nextafter(rho, 1.0);
      rho_out[l] = rho;
    }
  }
  return LAGS_OK;
}

int lags_last_routes(lags_ctx* ctx, const lags_table* t, int32_t* route, int32_t n) {
  if (!ctx || !t || t->ctx != ctx || !route || n != t->n) return LAGS_EINVAL;
  DeviceGuard g(ctx->device);
  if (!g.ok) return LAGS_EHIP;
  for (int32_t l = 0; l < n; ++l) route[l] = 0;
  const int nl = t->plan.n_large;
  if (nl == 0) return LAGS_OK;
  std::vector<LState> st;
  try {
    st.resize(nl);
  } catch (const std::bad_alloc&) {
    return LAGS_ENOMEM;
  }
  if (hipDeviceSynchronize() != hipSuccess) return LAGS_EHIP;
  if (hipMemcpy(st.data(), ctx->lstate.p, (size_t)nl * sizeof(LState), hipMemcpyDeviceToHost) != hipSuccess)
    return LAGS_EHIP;
  for (int i = 0; i < nl; ++i) route[t->lsegs[i].seg] = (int32_t)st[i].route;
  return LAGS_OK;
}

int lags_debug_fallback_chain(lags_ctx* ctx, int mode) {
  if (!ctx || mode < 0 || mode > 2) return LAGS_EINVAL;
  ctx->chain_mode = mode;
  ctx->armed_calls = 0;
  return LAGS_OK;
}

int lags_debug_scratch_info(lags_ctx* ctx, int which, const void** ptr, int64_t* bytes, int64_t* retired) {
  if (!ctx || !ptr || !bytes || !retired) return LAGS_EINVAL;
  const std::vector<DevBuf*> bufs = all_bufs(ctx);
  if (which < 0 || which >= (int)bufs.size()) return LAGS_EINVAL;
  *ptr = bufs[which]->p;
  *bytes = (int64_t)bufs[which]->bytes;
  *retired = (int64_t)ctx->retired.size();
  return LAGS_OK;
}

int lags_debug_poison_scratch(lags_ctx* ctx, void* hip_stream) {
  if (!ctx) return LAGS_EINVAL;
  DeviceGuard g(ctx->device);
  if (!g.ok) return LAGS_EHIP;
  for (DevBuf* b : all_bufs(ctx))
    if (b->p && launch_fill_u32(static_cast<uint32_t*>(b->p), (int64_t)(b->bytes / 4), 0xFFFFFFFFu,
                                (hipStream_t)hip_stream) != hipSuccess)
      return LAGS_EHIP;
  return LAGS_OK;
}

int lags_profile_enable(lags_ctx* ctx, int on) {
  if (!ctx) return LAGS_EINVAL;
  ctx->prof.on = on != 0;
  ctx->prof.only = -1;
  return LAGS_OK;
}

int lags_profile_enable_kernel(lags_ctx* ctx, int kernel_id) {
  if (!ctx || kernel_id < 0 || kernel_id >= K_NUM) return LAGS_EINVAL;
  ctx->prof.on = true;
  ctx->prof.only = kernel_id;
  return LAGS_OK;
}

int lags_profile_num_kernels(void) { return K_NUM; }

const char* lags_profile_kernel_name(int kernel_id) { return kernel_name(kernel_id); }

int lags_profile_read(lags_ctx* ctx, int kernel_id, double* total_ms, int64_t* launches) {
  if (!ctx || !total_ms || !launches || kernel_id < 0 || kernel_id >= K_NUM) return LAGS_EINVAL;
  DeviceGuard g(ctx->device);
  for (const Prof::Rec& r : ctx->prof.recs) {
    if (r.id != kernel_id) continue;
    float ms = 0.f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return LAGS_EHIP;
    *total_ms += (double)ms;
    *launches += r.launches;
  }
  return LAGS_OK;
}

int lags_profile_reset(lags_ctx* ctx) {
  if (!ctx) return LAGS_EINVAL;
  DeviceGuard g(ctx->device);
  for (const Prof::Rec& r : ctx->prof.recs) {
    (void)hipEventSynchronize(r.b);
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  ctx->prof.recs.clear();
  return LAGS_OK;
}

int64_t lags_profile_kernel_elements(const lags_table* t, int kernel_id) {
  if (!t) return -1;
  int64_t small[kSmallClasses] = {0, 0}, large = 0, all = 0;
  for (const SegDesc& sd : t->segs) {
    all += sd.d;
    if (sd.d <= kSmall0) small[0] += sd.d;
    else if (sd.d <= kSmall1) small[1] += sd.d;
    else large += sd.d;
  }
  switch (kernel_id) {
    case K_SMALL0: return small[0];
    case K_SMALL1: return small[1];
    case K_STREAM: return large;
    case K_MERGE: case K_MERGE_APPLY: case K_DELTA_TILES: case K_SPARSIFY_CALL: return all;
    default: return 0;
  }
}

const char* lags_strerror(int code) {
  switch (code) {
    case LAGS_OK: return "ok";
    case LAGS_EINVAL: return "invalid argument";
    case LAGS_ENOMEM: return "out of memory";
    case LAGS_EHIP: return "HIP runtime error";
    case LAGS_ECAPACITY: return "size beyond the library's capacity";
    default: return "unknown error";
  }
}

}  // extern "C"
