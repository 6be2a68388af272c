// HIP kernels (gfx950, wave64) of the per-layer error-compensated top-k sparsifier.
//
// What is computed (LAGS-SGD, Algorithm 1 lines 6-9, TopK of Eq. 4):
//   acc = residual + lr*grad; keep the k entries of largest |acc| (ties: lower index);
//   emit (index, acc) ascending; residual = acc with kept entries zeroed;
//   merge: update = (sum_p kept_p) / P.
//
// Selection is an exact radix select on key = bits(acc) & 0x7fffffff, digits of
// 11 + 10 + 10 bits from the top, with LDS histograms.  The k-th largest key T and the
// number r of entries equal to T that are still to be taken define the kept set:
// key > T, or key == T and fewer than r equal keys precede it in index order.
//
// Work layout: a wave owns a contiguous chunk of V*256 elements and walks it in V
// rounds; in a round lane i holds the 4 consecutive elements (round*256 + 4*i ..+3),
// so loads/stores are 16-byte vectors, coalesced over the wave, and index order is
// (round, lane, component).  Ordered compaction uses per-wave counts, a scan over waves
// (and over tiles for multi-block layers) and a wave prefix scan per round.
#include "lags_internal.h"

namespace lags {

// ------------------------------------------------------------------ helpers --
__device__ __forceinline__ int lane_id() {
  return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Algorithm 1 line 6 for one element: product rounded to binary32, then the sum
// rounded to binary32.  The empty asm keeps the two operations apart so that they
// can never be contracted into a fused multiply-add.
__device__ __forceinline__ uint32_t acc_bits(float g, float r, float lr) {
  float t = __fmul_rn(lr, g);
  asm volatile("" : "+v"(t));
  return __float_as_uint(__fadd_rn(r, t));
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t t = __shfl_up(x, o, 64);
    if (lane >= o) x += t;
  }
  return x;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

// Inclusive scan over the NT threads of the block; also returns the block total.
// s_wt must hold NT/64 entries.  Contains two barriers.
template <int NT>
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t v, uint32_t* s_wt, uint32_t& total) {
  constexpr int NW = NT / 64;
  const int lane = lane_id(), w = threadIdx.x >> 6;
  uint32_t x = wave_incl_scan(v, lane);
  __syncthreads();
  if (lane == 63) s_wt[w] = x;
  __syncthreads();
  uint32_t off = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    uint32_t t = s_wt[i];
    if (i < w) off += t;
    tot += t;
  }
  total = tot;
  return x + off;
}

// Given a histogram of `nb` bins (nb a multiple of NT) whose total is >= k_rem >= 1,
// find the bin b holding the k_rem-th entry counted from the top bin downwards and
// the rank of that entry inside the bin.  Result in s_sel[0] = b, s_sel[1] = new k_rem
// (valid for every thread after the call).  `hist` may be LDS or global memory.
template <int NT>
__device__ __forceinline__ void block_find_bucket(const uint32_t* hist, int nb, uint32_t k_rem,
                                                  uint32_t* s_wt, uint32_t* s_sel) {
  const int bpt = nb / NT;
  const int tid = threadIdx.x;
  uint32_t s = 0;
  for (int i = 0; i < bpt; ++i) s += hist[tid * bpt + i];
  uint32_t total;
  uint32_t incl = block_incl_scan<NT>(s, s_wt, total);
  uint32_t above = total - incl;  // entries in bins owned by higher threads
  if (above < k_rem && k_rem <= above + s) {
    uint32_t cum = above;
    for (int i = bpt - 1; i >= 0; --i) {
      uint32_t h = hist[tid * bpt + i];
      if (cum + h >= k_rem) {
        s_sel[0] = (uint32_t)(tid * bpt + i);
        s_sel[1] = k_rem - cum;
        break;
      }
      cum += h;
    }
  }
  __syncthreads();
}

// Load a wave's chunk of grad and residual and form acc (bits).  `n_w` = number of valid
// elements of the chunk counted from its start (may be <= 0 or > V*256).
template <int V>
__device__ __forceinline__ void load_acc(const float* __restrict__ g, const float* __restrict__ r,
                                         int n_w, float lr, bool vec, int lane, uint32_t (&a)[V][4]) {
  float4 gv[V], rv[V];
#pragma unroll
  for (int j = 0; j < V; ++j) {
    const int e = j * 256 + lane * 4;
    if (vec && e + 3 < n_w) {
      gv[j] = *reinterpret_cast<const float4*>(g + e);
      rv[j] = *reinterpret_cast<const float4*>(r + e);
    } else {
      gv[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      rv[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e + 0 < n_w) { gv[j].x = g[e + 0]; rv[j].x = r[e + 0]; }
      if (e + 1 < n_w) { gv[j].y = g[e + 1]; rv[j].y = r[e + 1]; }
      if (e + 2 < n_w) { gv[j].z = g[e + 2]; rv[j].z = r[e + 2]; }
      if (e + 3 < n_w) { gv[j].w = g[e + 3]; rv[j].w = r[e + 3]; }
    }
  }
#pragma unroll
  for (int j = 0; j < V; ++j) {
    a[j][0] = acc_bits(gv[j].x, rv[j].x, lr);
    a[j][1] = acc_bits(gv[j].y, rv[j].y, lr);
    a[j][2] = acc_bits(gv[j].z, rv[j].z, lr);
    a[j][3] = acc_bits(gv[j].w, rv[j].w, lr);
  }
}

// Load a wave's chunk of already formed acc values (bits).
template <int V>
__device__ __forceinline__ void load_bits(const float* __restrict__ r, int n_w, bool vec, int lane,
                                          uint32_t (&a)[V][4]) {
#pragma unroll
  for (int j = 0; j < V; ++j) {
    const int e = j * 256 + lane * 4;
    if (vec && e + 3 < n_w) {
      uint4 v = *reinterpret_cast<const uint4*>(r + e);
      a[j][0] = v.x; a[j][1] = v.y; a[j][2] = v.z; a[j][3] = v.w;
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) a[j][c] = (e + c < n_w) ? __float_as_uint(r[e + c]) : 0u;
    }
  }
}

template <int V>
__device__ __forceinline__ void store_bits(float* __restrict__ r, int n_w, bool vec, int lane,
                                           const uint32_t (&a)[V][4]) {
#pragma unroll
  for (int j = 0; j < V; ++j) {
    const int e = j * 256 + lane * 4;
    if (vec && e + 3 < n_w) {
      *reinterpret_cast<uint4*>(r + e) = make_uint4(a[j][0], a[j][1], a[j][2], a[j][3]);
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (e + c < n_w) r[e + c] = __uint_as_float(a[j][c]);
    }
  }
}

// Count, over a wave's chunk, the keys above T and equal to T (per-lane partial counts).
template <int V>
__device__ __forceinline__ void lane_count(const uint32_t (&a)[V][4], int n_w, int lane, uint32_t T,
                                           uint32_t& cg, uint32_t& ce) {
  cg = 0; ce = 0;
#pragma unroll
  for (int j = 0; j < V; ++j) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int e = j * 256 + lane * 4 + c;
      const uint32_t key = a[j][c] & 0x7FFFFFFFu;
      if (e < n_w) { cg += key > T; ce += key == T; }
    }
  }
}

// Ordered emission of a wave's chunk.  gt_before / eq_before: numbers of keys > T and
// == T that precede the chunk in the layer.  An element is kept if key > T, or key == T
// and fewer than `rtake` equal keys precede it; its output slot is the number of kept
// elements before it = gt_before + min(eq_before, rtake).
// FULL: the residual chunk is written completely (acc, kept entries zeroed).
// !FULL: the residual already holds acc; only the kept entries are zeroed.
template <int V, bool FULL>
__device__ __forceinline__ void wave_emit(uint32_t (&a)[V][4], int n_w, int lane, uint32_t T,
                                          uint32_t rtake, uint32_t gt_before, uint32_t eq_before,
                                          uint32_t k, int32_t idx_base, int32_t* __restrict__ oi,
                                          float* __restrict__ ov, float* __restrict__ r, bool vec) {
#pragma unroll
  for (int j = 0; j < V; ++j) {
    if (j * 256 >= n_w) break;  // wave-uniform
    const int e = j * 256 + lane * 4;
    uint32_t fg[4], fe[4];
    uint32_t ng = 0, ne = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t key = a[j][c] & 0x7FFFFFFFu;
      const bool valid = e + c < n_w;
      fg[c] = valid && key > T;
      fe[c] = valid && key == T;
      ng += fg[c];
      ne += fe[c];
    }
    const uint32_t packed = ng | (ne << 16);  // per round at most 256 each
    const uint32_t incl = wave_incl_scan(packed, lane);
    const uint32_t tot = __shfl(incl, 63, 64);
    const uint32_t excl = incl - packed;
    uint32_t gb = gt_before + (excl & 0xFFFFu);
    uint32_t eb = eq_before + (excl >> 16);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool sel = fg[c] || (fe[c] && eb < rtake);
      const uint32_t pos = gb + (eb < rtake ? eb : rtake);
      if (sel && pos < k) {  // pos < k always holds; the check keeps a wrong T from writing out of bounds
        oi[pos] = idx_base + e + c;
        ov[pos] = __uint_as_float(a[j][c]);
        if (FULL) a[j][c] = 0u; else r[e + c] = 0.0f;
      }
      gb += fg[c];
      eb += fe[c];
    }
    gt_before += tot & 0xFFFFu;
    eq_before += tot >> 16;
  }
  if (FULL) store_bits<V>(r, n_w, vec, lane, a);
}

__device__ __forceinline__ bool aligned16(const void* a, const void* b) {
  return ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15u) == 0;
}

// ------------------------------------------------------------------ zero -----
__global__ void k_zero_u32(uint32_t* __restrict__ p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) p[i] = 0u;
}

// ------------------------------------------------------------------ small ----
// One workgroup per layer; the layer's acc values live in registers from the single
// read of grad/residual to the single write of the residual.
template <int NW, int V>
__global__ __launch_bounds__(NW * 64) void k_small(const SegDesc* __restrict__ segs,
                                                   const int32_t* __restrict__ list,
                                                   const float* __restrict__ grad,
                                                   float* __restrict__ res, float lr,
                                                   int32_t* __restrict__ out_idx,
                                                   float* __restrict__ out_val) {
  constexpr int NT = NW * 64;
  constexpr int CH = V * 256;
  __shared__ uint32_t s_hist[kBins0];
  __shared__ uint32_t s_wt[NW];
  __shared__ uint32_t s_sel[2];
  __shared__ uint32_t s_wg[NW], s_we[NW];

  const SegDesc sd = segs[list[blockIdx.x]];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const float* g = grad + sd.offset + (int64_t)w * CH;
  float* r = res + sd.offset + (int64_t)w * CH;
  const int n_w = sd.d - w * CH;
  const bool vec = aligned16(g, r);

  uint32_t a[V][4];
  load_acc<V>(g, r, n_w, lr, vec, lane, a);

  uint32_t prefix = 0, mask = 0, k_rem = (uint32_t)sd.k;
#pragma unroll
  for (int level = 0; level < 3; ++level) {
    const int shift = level == 0 ? 20 : (level == 1 ? 10 : 0);
    const int nb = level == 0 ? kBins0 : kBins12;
    for (int i = tid; i < nb; i += NT) s_hist[i] = 0u;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < V; ++j) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int e = j * 256 + lane * 4 + c;
        const uint32_t key = a[j][c] & 0x7FFFFFFFu;
        if (e < n_w && (key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
      }
    }
    __syncthreads();
    block_find_bucket<NT>(s_hist, nb, k_rem, s_wt, s_sel);
    prefix |= s_sel[0] << shift;
    mask |= (uint32_t)(nb - 1) << shift;
    k_rem = s_sel[1];
    __syncthreads();
  }
  const uint32_t T = prefix, rtake = k_rem;

  uint32_t cg, ce;
  lane_count<V>(a, n_w, lane, T, cg, ce);
  cg = wave_sum(cg);
  ce = wave_sum(ce);
  if (lane == 0) { s_wg[w] = cg; s_we[w] = ce; }
  __syncthreads();
  uint32_t gb = 0, eb = 0;
  for (int i = 0; i < w; ++i) { gb += s_wg[i]; eb += s_we[i]; }
  wave_emit<V, true>(a, n_w, lane, T, rtake, gb, eb, (uint32_t)sd.k, w * CH, out_idx + sd.out_offset,
                     out_val + sd.out_offset, r, vec);
}

// ------------------------------------------------------------------ large ----
// Pass 1: acc = residual + lr*grad written into the residual buffer (it is the final
// residual everywhere but at the k kept entries), plus the histogram of key bits 30..20.
__global__ __launch_bounds__(256) void k_accum_hist(const TileDesc* __restrict__ tiles,
                                                    const float* __restrict__ grad,
                                                    float* __restrict__ res, float lr,
                                                    uint32_t* __restrict__ ghist) {
  __shared__ uint32_t s_hist[kBins0];
  const TileDesc td = tiles[blockIdx.x];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  for (int i = tid; i < kBins0; i += 256) s_hist[i] = 0u;
  const float* g = grad + td.start + w * kWaveChunk;
  float* r = res + td.start + w * kWaveChunk;
  const int n_w = td.n - w * kWaveChunk;
  const bool vec = aligned16(g, r);
  uint32_t a[kTileV][4];
  load_acc<kTileV>(g, r, n_w, lr, vec, lane, a);
  store_bits<kTileV>(r, n_w, vec, lane, a);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kTileV; ++j) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int e = j * 256 + lane * 4 + c;
      // Gradient magnitudes crowd into few bins: lanes that share lane 0's bin are
      // counted with one ballot and a single LDS add; the others add individually.
      const uint32_t b = e < n_w ? (a[j][c] & 0x7FFFFFFFu) >> 20 : 0xFFFFFFFFu;
      const uint32_t f = (uint32_t)__builtin_amdgcn_readfirstlane((int)b);
      const uint64_t same = __ballot(b == f);
      if (lane == 0 && f != 0xFFFFFFFFu) atomicAdd(&s_hist[f], (uint32_t)__popcll(same));
      if (b != f && b != 0xFFFFFFFFu) atomicAdd(&s_hist[b], 1u);
    }
  }
  __syncthreads();
  uint32_t* gh = ghist + (int64_t)td.seg * kHistStride;
  for (int i = tid; i < kBins0; i += 256) {
    const uint32_t h = s_hist[i];
    if (h) atomicAdd(&gh[i], h);
  }
}

// Decide one digit of T for every large layer from its histogram, then clear the
// histogram for the next pass.  One workgroup of 256 threads per layer.
__global__ __launch_bounds__(256) void k_choose(int level, const LargeSeg* __restrict__ lsegs,
                                                const SegDesc* __restrict__ segs,
                                                uint32_t* __restrict__ ghist,
                                                SegState* __restrict__ state) {
  __shared__ uint32_t s_wt[4];
  __shared__ uint32_t s_sel[2];
  const int ls = blockIdx.x;
  const int shift = level == 0 ? 20 : (level == 1 ? 10 : 0);
  const int nb = level == 0 ? kBins0 : kBins12;
  uint32_t* gh = ghist + (int64_t)ls * kHistStride;
  uint32_t prefix = 0, k_rem;
  if (level == 0) {
    k_rem = (uint32_t)segs[lsegs[ls].seg].k;
  } else {
    const SegState st = state[ls];
    prefix = st.prefix;
    k_rem = st.k_rem;
  }
  block_find_bucket<256>(gh, nb, k_rem, s_wt, s_sel);
  const uint32_t b = s_sel[0], kr = s_sel[1];
  __syncthreads();
  for (int i = threadIdx.x; i < nb; i += 256) gh[i] = 0u;
  if (threadIdx.x == 0) {
    SegState st;
    st.prefix = prefix | (b << shift);
    st.k_rem = kr;
    state[ls] = st;
  }
}

// Passes 2 and 3: histogram of the next 10 key bits over the entries whose higher
// bits equal the prefix decided so far.
template <int LEVEL>
__global__ __launch_bounds__(256) void k_hist(const TileDesc* __restrict__ tiles,
                                              const float* __restrict__ res,
                                              const SegState* __restrict__ state,
                                              uint32_t* __restrict__ ghist) {
  constexpr int shift = LEVEL == 1 ? 10 : 0;
  constexpr uint32_t mask = LEVEL == 1 ? 0x7FF00000u : 0x7FFFFC00u;
  __shared__ uint32_t s_hist[kBins12];
  const TileDesc td = tiles[blockIdx.x];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  for (int i = tid; i < kBins12; i += 256) s_hist[i] = 0u;
  const uint32_t prefix = state[td.seg].prefix;
  const float* r = res + td.start + w * kWaveChunk;
  const int n_w = td.n - w * kWaveChunk;
  const bool vec = aligned16(r, r);
  uint32_t a[kTileV][4];
  load_bits<kTileV>(r, n_w, vec, lane, a);
  __syncthreads();
  uint32_t any = 0;
#pragma unroll
  for (int j = 0; j < kTileV; ++j) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int e = j * 256 + lane * 4 + c;
      const uint32_t key = a[j][c] & 0x7FFFFFFFu;
      if (e < n_w && (key & mask) == prefix) {
        atomicAdd(&s_hist[(key >> shift) & (kBins12 - 1)], 1u);
        any = 1;
      }
    }
  }
  if (!__syncthreads_or((int)any)) return;
  uint32_t* gh = ghist + (int64_t)td.seg * kHistStride;
  for (int i = tid; i < kBins12; i += 256) {
    const uint32_t h = s_hist[i];
    if (h) atomicAdd(&gh[i], h);
  }
}

// With T known: per tile, how many keys are above T and how many equal T.
__global__ __launch_bounds__(256) void k_count(const TileDesc* __restrict__ tiles,
                                               const float* __restrict__ res,
                                               const SegState* __restrict__ state,
                                               uint32_t* __restrict__ tile_gt,
                                               uint32_t* __restrict__ tile_eq) {
  __shared__ uint32_t s_g[4], s_e[4];
  const TileDesc td = tiles[blockIdx.x];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const uint32_t T = state[td.seg].prefix;
  const float* r = res + td.start + w * kWaveChunk;
  const int n_w = td.n - w * kWaveChunk;
  uint32_t a[kTileV][4];
  load_bits<kTileV>(r, n_w, aligned16(r, r), lane, a);
  uint32_t cg, ce;
  lane_count<kTileV>(a, n_w, lane, T, cg, ce);
  cg = wave_sum(cg);
  ce = wave_sum(ce);
  if (lane == 0) { s_g[w] = cg; s_e[w] = ce; }
  __syncthreads();
  if (tid == 0) {
    tile_gt[blockIdx.x] = s_g[0] + s_g[1] + s_g[2] + s_g[3];
    tile_eq[blockIdx.x] = s_e[0] + s_e[1] + s_e[2] + s_e[3];
  }
}

// Exclusive scan of the per-tile counts inside each large layer (in place).
__global__ __launch_bounds__(256) void k_scan(const LargeSeg* __restrict__ lsegs,
                                              uint32_t* __restrict__ tile_gt,
                                              uint32_t* __restrict__ tile_eq) {
  __shared__ uint32_t s_wt[4];
  const LargeSeg ls = lsegs[blockIdx.x];
  uint32_t carry_g = 0, carry_e = 0;
  for (int base = ls.tile_begin; base < ls.tile_end; base += 256) {
    const int i = base + threadIdx.x;
    const uint32_t vg = i < ls.tile_end ? tile_gt[i] : 0u;
    const uint32_t ve = i < ls.tile_end ? tile_eq[i] : 0u;
    uint32_t tg, te;
    const uint32_t ig = block_incl_scan<256>(vg, s_wt, tg);
    const uint32_t ie = block_incl_scan<256>(ve, s_wt, te);
    if (i < ls.tile_end) {
      tile_gt[i] = carry_g + ig - vg;
      tile_eq[i] = carry_e + ie - ve;
    }
    carry_g += tg;
    carry_e += te;
  }
}

// Final pass: ordered emission of the kept pairs and zeroing of their residual slots.
__global__ __launch_bounds__(256) void k_emit(const TileDesc* __restrict__ tiles,
                                              const LargeSeg* __restrict__ lsegs,
                                              const SegDesc* __restrict__ segs,
                                              float* __restrict__ res,
                                              const SegState* __restrict__ state,
                                              const uint32_t* __restrict__ tile_gt,
                                              const uint32_t* __restrict__ tile_eq,
                                              int32_t* __restrict__ out_idx,
                                              float* __restrict__ out_val) {
  __shared__ uint32_t s_g[4], s_e[4];
  const TileDesc td = tiles[blockIdx.x];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const SegState st = state[td.seg];
  const uint32_t T = st.prefix, rtake = st.k_rem;
  const uint32_t tg = tile_gt[blockIdx.x], te = tile_eq[blockIdx.x];
  const SegDesc sd = segs[lsegs[td.seg].seg];
  const int64_t out_off = sd.out_offset;
  float* r = res + td.start + w * kWaveChunk;
  const int n_w = td.n - w * kWaveChunk;
  const bool vec = aligned16(r, r);
  uint32_t a[kTileV][4];
  load_bits<kTileV>(r, n_w, vec, lane, a);
  uint32_t cg, ce;
  lane_count<kTileV>(a, n_w, lane, T, cg, ce);
  cg = wave_sum(cg);
  ce = wave_sum(ce);
  if (lane == 0) { s_g[w] = cg; s_e[w] = ce; }
  __syncthreads();
  uint32_t gb = tg, eb = te;
  for (int i = 0; i < w; ++i) { gb += s_g[i]; eb += s_e[i]; }
  // nothing to emit in this wave if it holds no key above T and its ties come too late
  if (cg == 0 && (ce == 0 || eb >= rtake)) return;
  wave_emit<kTileV, false>(a, n_w, lane, T, rtake, gb, eb, (uint32_t)sd.k, td.local0 + w * kWaveChunk,
                           out_idx + out_off, out_val + out_off, r, vec);
}

// ------------------------------------------------------------------ merge ----
// Algorithm 1 lines 8-9.  One workgroup owns one tile of the dense update: it
// accumulates the tile in LDS, adding the workers' entries in worker order (a barrier
// between workers; inside one worker the indices are distinct), then writes the tile
// once, divided by P.  No atomics, fixed summation order.
__global__ __launch_bounds__(256) void k_merge(const TileDesc* __restrict__ mtiles,
                                               const SegDesc* __restrict__ segs,
                                               const int32_t* __restrict__ idx,
                                               const float* __restrict__ val, int P,
                                               int64_t stride_k, float* __restrict__ update) {
  __shared__ float s_acc[kMergeTile];
  __shared__ int32_t s_lo[64], s_hi[64];
  const TileDesc td = mtiles[blockIdx.x];
  const SegDesc sd = segs[td.seg];
  const int tid = threadIdx.x;
  for (int i = tid; i < kMergeTile; i += 256) s_acc[i] = 0.0f;
  for (int p0 = 0; p0 < P; p0 += 64) {
    const int np = P - p0 < 64 ? P - p0 : 64;
    __syncthreads();
    if (tid < 2 * np) {
      // first position in worker p's index list of this layer that is >= target
      const int p = p0 + (tid >> 1);
      const int32_t target = td.local0 + ((tid & 1) ? td.n : 0);
      const int32_t* li = idx + (int64_t)p * stride_k + sd.out_offset;
      int lo = 0, hi = sd.k;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (li[mid] < target) lo = mid + 1; else hi = mid;
      }
      if (tid & 1) s_hi[tid >> 1] = lo; else s_lo[tid >> 1] = lo;
    }
    __syncthreads();
    for (int q = 0; q < np; ++q) {
      const int64_t base = (int64_t)(p0 + q) * stride_k + sd.out_offset;
      const int hi = s_hi[q];
      for (int j = s_lo[q] + tid; j < hi; j += 256) {
        const uint32_t off = (uint32_t)(idx[base + j] - td.local0);
        if (off < (uint32_t)td.n) s_acc[off] = __fadd_rn(s_acc[off], val[base + j]);
      }
      __syncthreads();
    }
  }
  const float fp = (float)P;
  float* u = update + td.start;
  const bool vec = aligned16(u, u);
  for (int e = tid * 4; e < td.n; e += 1024) {
    if (vec && e + 3 < td.n) {
      float4 v;
      v.x = __fdiv_rn(s_acc[e + 0], fp);
      v.y = __fdiv_rn(s_acc[e + 1], fp);
      v.z = __fdiv_rn(s_acc[e + 2], fp);
      v.w = __fdiv_rn(s_acc[e + 3], fp);
      *reinterpret_cast<float4*>(u + e) = v;
    } else {
      for (int c = 0; c < 4; ++c)
        if (e + c < td.n) u[e + c] = __fdiv_rn(s_acc[e + c], fp);
    }
  }
}

// ------------------------------------------------------------------ launch ---
const char* kernel_name(int id) {
  static const char* names[K_NUM] = {"k_zero_u32", "k_small<4,1>", "k_small<4,8>", "k_small<16,10>",
                                     "k_accum_hist", "k_choose", "k_hist", "k_count", "k_scan", "k_emit",
                                     "k_merge"};
  return (id >= 0 && id < K_NUM) ? names[id] : nullptr;
}

hipError_t launch_zero_u32(uint32_t* p, int64_t n, hipStream_t s, Prof* prof) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  ProfScope ps(prof, K_ZERO, s);
  hipLaunchKernelGGL(k_zero_u32, dim3((unsigned)blocks), dim3(256), 0, s, p, n);
  return hipGetLastError();
}

hipError_t launch_small(int cls, int nseg, const SegDesc* segs, const int32_t* list, const float* grad,
                        float* res, float lr, int32_t* out_idx, float* out_val, hipStream_t s, Prof* prof) {
  if (nseg <= 0) return hipSuccess;
  ProfScope ps(prof, K_SMALL0 + cls, s);
  if (cls == 0)
    hipLaunchKernelGGL((k_small<4, 1>), dim3(nseg), dim3(256), 0, s, segs, list, grad, res, lr, out_idx, out_val);
  else if (cls == 1)
    hipLaunchKernelGGL((k_small<4, 8>), dim3(nseg), dim3(256), 0, s, segs, list, grad, res, lr, out_idx, out_val);
  else
    hipLaunchKernelGGL((k_small<16, 10>), dim3(nseg), dim3(1024), 0, s, segs, list, grad, res, lr, out_idx, out_val);
  return hipGetLastError();
}

hipError_t launch_large(int n_large, int n_tiles, const SegDesc* segs, const LargeSeg* lsegs,
                        const TileDesc* tiles, const float* grad, float* res, float lr,
                        int32_t* out_idx, float* out_val, uint32_t* ghist, SegState* state,
                        uint32_t* tile_gt, uint32_t* tile_eq, hipStream_t s, Prof* prof) {
  if (n_large <= 0) return hipSuccess;
  hipError_t e = launch_zero_u32(ghist, (int64_t)n_large * kHistStride, s, prof);
  if (e != hipSuccess) return e;
  {
    ProfScope ps(prof, K_ACCUM_HIST, s);
    hipLaunchKernelGGL(k_accum_hist, dim3(n_tiles), dim3(256), 0, s, tiles, grad, res, lr, ghist);
  }
  for (int level = 0; level < 3; ++level) {
    if (level == 1) {
      ProfScope ps(prof, K_HIST, s);
      hipLaunchKernelGGL(k_hist<1>, dim3(n_tiles), dim3(256), 0, s, tiles, res, state, ghist);
    } else if (level == 2) {
      ProfScope ps(prof, K_HIST, s);
      hipLaunchKernelGGL(k_hist<2>, dim3(n_tiles), dim3(256), 0, s, tiles, res, state, ghist);
    }
    ProfScope ps(prof, K_CHOOSE, s);
    hipLaunchKernelGGL(k_choose, dim3(n_large), dim3(256), 0, s, level, lsegs, segs, ghist, state);
  }
  {
    ProfScope ps(prof, K_COUNT, s);
    hipLaunchKernelGGL(k_count, dim3(n_tiles), dim3(256), 0, s, tiles, res, state, tile_gt, tile_eq);
  }
  {
    ProfScope ps(prof, K_SCAN, s);
    hipLaunchKernelGGL(k_scan, dim3(n_large), dim3(256), 0, s, lsegs, tile_gt, tile_eq);
  }
  {
    ProfScope ps(prof, K_EMIT, s);
    hipLaunchKernelGGL(k_emit, dim3(n_tiles), dim3(256), 0, s, tiles, lsegs, segs, res, state, tile_gt,
                       tile_eq, out_idx, out_val);
  }
  return hipGetLastError();
}

hipError_t launch_merge(int n_tiles, const TileDesc* mtiles, const SegDesc* segs, const int32_t* idx,
                        const float* val, int P, int64_t stride_k, float* update, hipStream_t s, Prof* prof) {
  if (n_tiles <= 0) return hipSuccess;
  ProfScope ps(prof, K_MERGE, s);
  hipLaunchKernelGGL(k_merge, dim3(n_tiles), dim3(256), 0, s, mtiles, segs, idx, val, P, stride_k, update);
  return hipGetLastError();
}

}  // namespace lags
