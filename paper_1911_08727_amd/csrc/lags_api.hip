// Host side of liblags.so: the C ABI declared in include/lags.h.
// Validates arguments, prepares layer tables (k per layer, output positions, size
// classes, tile lists), owns the scratch arena and enqueues the kernels.
#include "../../include/lags.h"
#include "lags_internal.h"

#include <algorithm>
#include <cmath>
#include <map>
#include <new>
#include <utility>
#include <vector>

using namespace lags;

struct lags_ctx {
  int device = 0;
  // scratch of the multi-block path, sized for the largest table created so far
  uint32_t* ghist = nullptr;   int64_t ghist_cap = 0;    // n_large * kHistStride
  SegState* state = nullptr;   int64_t state_cap = 0;    // n_large
  uint32_t* tile_gt = nullptr; uint32_t* tile_eq = nullptr; int64_t tile_cap = 0;  // n_tiles
  std::map<std::pair<int64_t, int64_t>, lags_table*> layer_tables;  // (d, k) -> one-layer table
  Prof prof;
};

struct lags_table {
  lags_ctx* ctx = nullptr;
  int32_t n = 0;
  int64_t total_k = 0;
  int64_t span_lo = 0, span_hi = 0;            // [min offset, max offset + d)
  std::vector<SegDesc> segs;                   // host copy
  int n_small[3] = {0, 0, 0};
  int n_large = 0, n_tiles = 0, n_mtiles = 0;
  SegDesc* d_segs = nullptr;
  int32_t* d_small[3] = {nullptr, nullptr, nullptr};
  LargeSeg* d_lsegs = nullptr;
  TileDesc* d_tiles = nullptr;
  TileDesc* d_mtiles = nullptr;
};

namespace {

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

template <typename T>
int grow(T** p, int64_t* cap, int64_t need) {
  if (need <= *cap) return LAGS_OK;
  if (*p) (void)hipFree(*p);
  *p = nullptr;
  *cap = 0;
  if (hipMalloc(reinterpret_cast<void**>(p), (size_t)need * sizeof(T)) != hipSuccess) {
    *p = nullptr;
    return LAGS_ENOMEM;
  }
  *cap = need;
  return LAGS_OK;
}

bool ranges_overlap(const void* a, int64_t abytes, const void* b, int64_t bbytes) {
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a0 < b0 + (uintptr_t)bbytes && b0 < a0 + (uintptr_t)abytes;
}

void free_table_device(lags_table* t) {
  if (t->d_segs) (void)hipFree(t->d_segs);
  for (int c = 0; c < 3; ++c)
    if (t->d_small[c]) (void)hipFree(t->d_small[c]);
  if (t->d_lsegs) (void)hipFree(t->d_lsegs);
  if (t->d_tiles) (void)hipFree(t->d_tiles);
  if (t->d_mtiles) (void)hipFree(t->d_mtiles);
}

// Build a table from explicit (offset, d, k) triples.
int build_table(lags_ctx* ctx, const std::vector<int64_t>& off, const std::vector<int64_t>& d,
                const std::vector<int64_t>& k, lags_table** out) {
  const int32_t n = (int32_t)off.size();
  lags_table* t = new (std::nothrow) lags_table();
  if (!t) return LAGS_ENOMEM;
  t->ctx = ctx;
  t->n = n;
  std::vector<int32_t> small[3];
  std::vector<LargeSeg> lsegs;
  std::vector<TileDesc> tiles, mtiles;
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
      else if (d[l] <= kSmall2) small[2].push_back(l);
      else {
        LargeSeg ls;
        ls.seg = l;
        ls.tile_begin = (int32_t)tiles.size();
        const int64_t nt = (d[l] + kTile - 1) / kTile;
        if ((int64_t)tiles.size() + nt > 0x3FFFFFFF) { delete t; return LAGS_ECAPACITY; }
        for (int64_t i = 0; i < nt; ++i) {
          TileDesc td;
          td.start = off[l] + i * kTile;
          td.n = (int32_t)std::min<int64_t>(kTile, d[l] - i * kTile);
          td.seg = (int32_t)lsegs.size();
          td.local0 = (int32_t)(i * kTile);
          td.pad = 0;
          tiles.push_back(td);
        }
        ls.tile_end = (int32_t)tiles.size();
        ls.pad = 0;
        lsegs.push_back(ls);
      }
      const int64_t nmt = (d[l] + kMergeTile - 1) / kMergeTile;
      if ((int64_t)mtiles.size() + nmt > 0x3FFFFFFF) { delete t; return LAGS_ECAPACITY; }
      for (int64_t i = 0; i < nmt; ++i) {
        TileDesc td;
        td.start = off[l] + i * kMergeTile;
        td.n = (int32_t)std::min<int64_t>(kMergeTile, d[l] - i * kMergeTile);
        td.seg = l;
        td.local0 = (int32_t)(i * kMergeTile);
        td.pad = 0;
        mtiles.push_back(td);
      }
    }
    t->total_k = outpos;
  } catch (const std::bad_alloc&) {
    delete t;
    return LAGS_ENOMEM;
  }
  for (int c = 0; c < 3; ++c) t->n_small[c] = (int)small[c].size();
  t->n_large = (int)lsegs.size();
  t->n_tiles = (int)tiles.size();
  t->n_mtiles = (int)mtiles.size();

  int rc = upload(&t->d_segs, t->segs);
  for (int c = 0; c < 3 && rc == LAGS_OK; ++c) rc = upload(&t->d_small[c], small[c]);
  if (rc == LAGS_OK) rc = upload(&t->d_lsegs, lsegs);
  if (rc == LAGS_OK) rc = upload(&t->d_tiles, tiles);
  if (rc == LAGS_OK) rc = upload(&t->d_mtiles, mtiles);
  if (rc == LAGS_OK) rc = grow(&ctx->ghist, &ctx->ghist_cap, (int64_t)t->n_large * kHistStride);
  if (rc == LAGS_OK) rc = grow(&ctx->state, &ctx->state_cap, (int64_t)t->n_large);
  if (rc == LAGS_OK && t->n_tiles > ctx->tile_cap) {
    if (ctx->tile_gt) (void)hipFree(ctx->tile_gt);
    if (ctx->tile_eq) (void)hipFree(ctx->tile_eq);
    ctx->tile_gt = ctx->tile_eq = nullptr;
    ctx->tile_cap = 0;
    int64_t c1 = 0, c2 = 0;
    rc = grow(&ctx->tile_gt, &c1, t->n_tiles);
    if (rc == LAGS_OK) rc = grow(&ctx->tile_eq, &c2, t->n_tiles);
    if (rc == LAGS_OK) ctx->tile_cap = t->n_tiles;
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
  for (int c = 0; c < 3; ++c) {
    if (launch_small(c, t->n_small[c], t->d_segs, t->d_small[c], grad, res, lr, out_idx, out_val, s, &ctx->prof) != hipSuccess)
      return LAGS_EHIP;
  }
  if (launch_large(t->n_large, t->n_tiles, t->d_segs, t->d_lsegs, t->d_tiles, grad, res, lr, out_idx,
                   out_val, ctx->ghist, ctx->state, ctx->tile_gt, ctx->tile_eq, s, &ctx->prof) != hipSuccess)
    return LAGS_EHIP;
  return LAGS_OK;
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
  *out = c;
  return LAGS_OK;
}

int lags_destroy(lags_ctx* ctx) {
  if (!ctx) return LAGS_EINVAL;
  DeviceGuard g(ctx->device);
  (void)lags_profile_reset(ctx);
  for (auto& kv : ctx->layer_tables) {
    free_table_device(kv.second);
    delete kv.second;
  }
  if (ctx->ghist) (void)hipFree(ctx->ghist);
  if (ctx->state) (void)hipFree(ctx->state);
  if (ctx->tile_gt) (void)hipFree(ctx->tile_gt);
  if (ctx->tile_eq) (void)hipFree(ctx->tile_eq);
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

int lags_merge_sparse(lags_ctx* ctx, const lags_table* t, const int32_t* idx, const float* val, int32_t P,
                      int64_t stride_k, float* update_flat, void* hip_stream) {
  if (!ctx || !t || t->ctx != ctx || !idx || !val || !update_flat) return LAGS_EINVAL;
  if (P < 1 || P > kMaxWorkers || stride_k < t->total_k) return LAGS_EINVAL;
  const int64_t pb = ((int64_t)(P - 1) * stride_k + t->total_k) * 4;
  const char* up = reinterpret_cast<const char*>(update_flat) + t->span_lo * 4;
  const int64_t ub = (t->span_hi - t->span_lo) * 4;
  if (ranges_overlap(up, ub, idx, pb) || ranges_overlap(up, ub, val, pb)) return LAGS_EINVAL;
  DeviceGuard g(ctx->device);
  if (!g.ok) return LAGS_EHIP;
  if (launch_merge(t->n_mtiles, t->d_mtiles, t->d_segs, idx, val, P, stride_k, update_flat,
                   (hipStream_t)hip_stream, &ctx->prof) != hipSuccess)
    return LAGS_EHIP;
  return LAGS_OK;
}

int lags_profile_enable(lags_ctx* ctx, int on) {
  if (!ctx) return LAGS_EINVAL;
  ctx->prof.on = on != 0;
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
    *launches += 1;
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
  int64_t small[3] = {0, 0, 0}, large = 0, all = 0;
  for (const SegDesc& sd : t->segs) {
    all += sd.d;
    if (sd.d <= kSmall0) small[0] += sd.d;
    else if (sd.d <= kSmall1) small[1] += sd.d;
    else if (sd.d <= kSmall2) small[2] += sd.d;
    else large += sd.d;
  }
  switch (kernel_id) {
    case K_SMALL0: return small[0];
    case K_SMALL1: return small[1];
    case K_SMALL2: return small[2];
    case K_ACCUM_HIST: case K_HIST: case K_COUNT: case K_EMIT: return large;
    case K_MERGE: return all;
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
