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
//
// Three routes, chosen per layer by size:
//   small  (d <= 40960): one workgroup, acc stays in registers between the single read of
//          grad/residual and the single write of the residual.
//   large, sampled: a sample of 16384 elements gives a threshold tau that, with high
//          probability, admits slightly more than k entries.  One streaming pass writes acc
//          into the residual buffer and collects every entry with key >= tau (in index
//          order).  If at least k were collected (and the lists did not overflow) the exact
//          top k are among them and the selection runs on the short candidate list only.
//          The guess never changes the result: it is verified by the count.
//   large, fallback: radix select over the acc values in the residual buffer, multi-block.
#include "lags_internal.h"

namespace lags {

// ------------------------------------------------------------------ helpers --
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int lane_id() {
  return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// number of set bits of `m` below the calling lane
__device__ __forceinline__ uint32_t mbcnt64(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
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
// (valid for every thread after the call; untouched if the total is below k_rem).
// `hist` may be LDS or global memory.
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

// Histogram update where many lanes may hit the same bin: lanes that share lane 0's bin
// are counted with one ballot and a single LDS add; the others add individually.
// b = 0xFFFFFFFF: the lane has nothing to add.  Must be called by all 64 lanes.
__device__ __forceinline__ void hist_add_peeled(uint32_t* s_hist, uint32_t b, int lane) {
  const uint32_t f = (uint32_t)__builtin_amdgcn_readfirstlane((int)b);
  const uint64_t same = __ballot(b == f);
  if (lane == 0 && f != 0xFFFFFFFFu) atomicAdd(&s_hist[f], (uint32_t)__popcll(same));
  if (b != f && b != 0xFFFFFFFFu) atomicAdd(&s_hist[b], 1u);
}

// Exact radix select over keys held in registers by a whole workgroup: finds the k-th
// largest key T and the number of entries equal to T that belong to the top k.
// s_hist: kBins0 words, s_wt: NT/64 words, s_sel: 2 words.
// Entries with key < floor_key are left out: the result is the same as long as at least k
// entries reach the floor (a caller that knows a lower bound of T saves their histogram adds).
// If fewer than k entries take part, T = 0 and rtake = 0 are returned.
template <int NT, int V>
__device__ __forceinline__ void block_radix_select(const uint32_t (&a)[V][4], int n_w, int lane, uint32_t k,
                                                   uint32_t* s_hist, uint32_t* s_wt, uint32_t* s_sel,
                                                   uint32_t& T, uint32_t& rtake, uint32_t floor_key = 0u) {
  const int tid = threadIdx.x;
  uint32_t prefix = 0, mask = 0, k_rem = k;
#pragma unroll
  for (int level = 0; level < 3; ++level) {
    const int shift = level == 0 ? 20 : (level == 1 ? 10 : 0);
    const int nb = level == 0 ? kBins0 : kBins12;
    for (int i = tid; i < nb; i += NT) s_hist[i] = 0u;
    if (tid == 0) { s_sel[0] = 0u; s_sel[1] = 0u; }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < V; ++j) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int e = j * 256 + lane * 4 + c;
        const uint32_t key = a[j][c] & 0x7FFFFFFFu;
        if (e < n_w && key >= floor_key && (key & mask) == prefix)
          atomicAdd(&s_hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
      }
    }
    __syncthreads();
    block_find_bucket<NT>(s_hist, nb, k_rem, s_wt, s_sel);
    prefix |= s_sel[0] << shift;
    mask |= (uint32_t)(nb - 1) << shift;
    k_rem = s_sel[1];
    __syncthreads();
  }
  T = prefix;
  rtake = k_rem;
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

// Load the value bits of a wave's chunk of a candidate list ((index, bits) pairs).
template <int V>
__device__ __forceinline__ void load_cand_bits(const uint2* __restrict__ cw, int n_w, int lane,
                                               uint32_t (&a)[V][4]) {
#pragma unroll
  for (int j = 0; j < V; ++j) {
    const int e = j * 256 + lane * 4;
#pragma unroll
    for (int c = 0; c < 4; ++c) a[j][c] = (e + c < n_w) ? cw[e + c].y : 0u;
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

enum { EMIT_FULL = 0, EMIT_ZERO = 1, EMIT_CAND = 2 };

// Ordered emission of a wave's chunk.  gt_before / eq_before: numbers of keys > T and
// == T that precede the chunk in the layer.  An element is kept if key > T, or key == T
// and fewer than `rtake` equal keys precede it; its output slot is the number of kept
// elements before it = gt_before + min(eq_before, rtake).
// EMIT_FULL: the chunk is residual data; it is written back completely (acc, kept entries
//            zeroed).  r = the chunk's residual.
// EMIT_ZERO: the residual already holds acc; only the kept entries are zeroed.  r = the
//            chunk's residual.
// EMIT_CAND: the chunk is part of a candidate list cw ((index, bits) pairs).  The streaming
//            pass already wrote zero for the entries with key >= tau_hi and acc for the others,
//            so r[index] is written only where that differs from the outcome: zero for kept
//            entries below tau_hi, acc for dropped entries at or above it.  r = the layer's residual.
template <int V, int MODE>
__device__ __forceinline__ void wave_emit(uint32_t (&a)[V][4], int n_w, int lane, uint32_t T,
                                          uint32_t rtake, uint32_t gt_before, uint32_t eq_before,
                                          uint32_t k, int32_t idx_base, int32_t* __restrict__ oi,
                                          float* __restrict__ ov, float* __restrict__ r, bool vec,
                                          const uint2* __restrict__ cw, uint32_t tau_hi) {
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
      if (MODE == EMIT_CAND) {
        const bool zeroed = (a[j][c] & 0x7FFFFFFFu) >= tau_hi;  // what the streaming pass assumed
        if (e + c < n_w && (sel || zeroed)) {
          const int32_t index = (int32_t)cw[e + c].x;
          if (sel && pos < k) {  // pos < k always holds; the check keeps a wrong T from writing out of bounds
            ov[pos] = __uint_as_float(a[j][c]);
            oi[pos] = index;
          }
          if (sel && !zeroed) r[index] = 0.0f;
          if (!sel && zeroed) r[index] = __uint_as_float(a[j][c]);
        }
      } else if (sel && pos < k) {
        ov[pos] = __uint_as_float(a[j][c]);
        oi[pos] = idx_base + e + c;
        if (MODE == EMIT_FULL) a[j][c] = 0u; else r[e + c] = 0.0f;
      }
      gb += fg[c];
      eb += fe[c];
    }
    gt_before += tot & 0xFFFFu;
    eq_before += tot >> 16;
  }
  if (MODE == EMIT_FULL) store_bits<V>(r, n_w, vec, lane, a);
}

__device__ __forceinline__ bool aligned16(const void* a, const void* b) {
  return ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15u) == 0;
}

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// ------------------------------------------------------------------ zero -----
__global__ void k_zero_u32(uint32_t* __restrict__ p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) p[i] = 0u;
}

// ------------------------------------------------------------------ small ----
// One workgroup per layer (CAND = false) or per candidate list of a large layer
// (CAND = true); the values live in registers between the single read and the write.
template <int NW, int V, bool CAND>
__global__ __launch_bounds__(NW * 64) void k_small(const SegDesc* __restrict__ segs,
                                                   const int32_t* __restrict__ list,
                                                   const LargeSeg* __restrict__ lsegs,
                                                   const LState* __restrict__ lstate,
                                                   const uint2* __restrict__ cand,
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

  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  SegDesc sd;
  int n;
  const uint2* cw = nullptr;
  uint32_t tau_hi = 0xFFFFFFFFu;
  if (CAND) {
    const int li = list[blockIdx.x];
    const LargeSeg ls = lsegs[li];
    const LState st = lstate[li];
    if (st.mode != MODE_SPARSE) return;  // uniform over the workgroup
    tau_hi = st.tau_hi;
    sd = segs[ls.seg];
    n = (int)st.ncand;
    cw = cand + ls.cand_base + (int64_t)w * CH;
  } else {
    sd = segs[list[blockIdx.x]];
    n = sd.d;
  }
  const int n_w = n - w * CH;
  float* r = res + sd.offset + (int64_t)w * CH;
  bool vec = false;

  uint32_t a[V][4];
  if (CAND) {
    load_cand_bits<V>(cw, n_w, lane, a);
  } else {
    const float* g = grad + sd.offset + (int64_t)w * CH;
    vec = aligned16(g, r);
    load_acc<V>(g, r, n_w, lr, vec, lane, a);
  }

  uint32_t T, rtake;
  block_radix_select<NT, V>(a, n_w, lane, (uint32_t)sd.k, s_hist, s_wt, s_sel, T, rtake);

  uint32_t cg, ce;
  lane_count<V>(a, n_w, lane, T, cg, ce);
  cg = wave_sum(cg);
  ce = wave_sum(ce);
  if (lane == 0) { s_wg[w] = cg; s_we[w] = ce; }
  __syncthreads();
  uint32_t gb = 0, eb = 0;
  for (int i = 0; i < w; ++i) { gb += s_wg[i]; eb += s_we[i]; }
  if (CAND)
    wave_emit<V, EMIT_CAND>(a, n_w, lane, T, rtake, gb, eb, (uint32_t)sd.k, 0, out_idx + sd.out_offset,
                            out_val + sd.out_offset, res + sd.offset, false, cw, tau_hi);
  else
    wave_emit<V, EMIT_FULL>(a, n_w, lane, T, rtake, gb, eb, (uint32_t)sd.k, w * CH, out_idx + sd.out_offset,
                            out_val + sd.out_offset, r, vec, nullptr, 0u);
}

// ------------------------------------------------------------------ sample ---
// Threshold guess for one large layer: form acc on up to 256 pieces of 64 (V = 4) or 256
// (V = 16) consecutive elements spread over the layer (with a hashed offset inside each
// stride), and take the sample's `sample_rank`-th largest key as tau and its
// `sample_rank_hi`-th largest (the sample's estimate of the layer's k-th largest) as tau_hi.
// Missing sample slots count as key 0.
template <int V>
__device__ __forceinline__ void sample_layer(const LargeSeg& ls, int li, const SegDesc& sd,
                                             const float* __restrict__ grad, const float* __restrict__ res,
                                             float lr, LState* __restrict__ lstate, uint32_t* s_hist,
                                             uint32_t* s_wt, uint32_t* s_sel) {
  constexpr int NT = 1024;  // 16 waves; a wave takes 4 pieces per round
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const float* g = grad + sd.offset;
  const float* r = res + sd.offset;
  const bool vec = aligned16(g, r);
  // V = 4: a round of a wave covers 4 pieces of 64 elements (16 lanes each); the large sample
  // (V = 16) takes the same number of pieces, each 256 elements long (one wave round), so that
  // it touches no more pages than the small one
  constexpr int PL = V == 4 ? kSamplePiece : 256;       // piece length
  constexpr int LP = PL / 4;                            // lanes per piece
  constexpr int PR = 64 / LP;                           // pieces per wave round
  uint32_t a[V][4];
#pragma unroll
  for (int j = 0; j < V; ++j) {
    const int piece = w * (V * PR) + j * PR + (lane / LP);
    a[j][0] = a[j][1] = a[j][2] = a[j][3] = 0u;
    if (piece < ls.sample_pieces) {
      int start = piece * ls.sample_stride;
      if (ls.sample_stride > PL)
        start += (int)(mix32((uint32_t)piece * 0x9E3779B9u + (uint32_t)li) % (uint32_t)(ls.sample_stride - PL + 1));
      start &= ~3;
      const int e = start + (lane % LP) * 4;
      if (vec && e + 3 < sd.d) {
        const float4 gv = *reinterpret_cast<const float4*>(g + e);
        const float4 rv = *reinterpret_cast<const float4*>(r + e);
        a[j][0] = acc_bits(gv.x, rv.x, lr);
        a[j][1] = acc_bits(gv.y, rv.y, lr);
        a[j][2] = acc_bits(gv.z, rv.z, lr);
        a[j][3] = acc_bits(gv.w, rv.w, lr);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (e + c < sd.d) a[j][c] = acc_bits(g[e + c], r[e + c], lr);
      }
    }
  }
  // The large sample first finds a lower bound of the rank-j key, so that the selections below
  // add a few hundred entries to their histograms instead of 65536 whose exponents share a
  // handful of LDS bins (measured 2.5x faster on normal data; not worth its own selection for
  // the small sample): the j-th largest of the 1024 per-thread maxima is the j-th largest of a
  // subset of the sample.
  uint32_t floor_key = 0u, rtake;
  if (V == 16 && ls.sample_rank <= NT) {  // uniform over the workgroup
    uint32_t mx[1][4] = {{0u, 0u, 0u, 0u}};
#pragma unroll
    for (int j = 0; j < V; ++j) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t key = a[j][c] & 0x7FFFFFFFu;
        mx[0][0] = key > mx[0][0] ? key : mx[0][0];
      }
    }
    // one value per thread in component 0; the empty components (key 0) stay below the floor 1
    block_radix_select<NT, 1>(mx, 256, lane, (uint32_t)ls.sample_rank, s_hist, s_wt, s_sel, floor_key, rtake, 1u);
  }
  uint32_t T, Thi = 0xFFFFFFFFu;
  block_radix_select<NT, V>(a, V * 256, lane, (uint32_t)ls.sample_rank, s_hist, s_wt, s_sel, T, rtake, floor_key);
  if (ls.sample_rank_hi > 0)  // uniform over the workgroup
    block_radix_select<NT, V>(a, V * 256, lane, (uint32_t)ls.sample_rank_hi, s_hist, s_wt, s_sel, Thi, rtake,
                              floor_key);
  if (tid == 0) {
    lstate[li].tau = T;
    lstate[li].tau_hi = Thi;  // >= T because sample_rank_hi <= sample_rank
  }
}

// One workgroup per sampled layer.  BIG: the table holds layers with the large sample; those
// workgroups take the V = 16 path.
template <bool BIG>
__global__ __launch_bounds__(1024) void k_sample(const SegDesc* __restrict__ segs,
                                                 const int32_t* __restrict__ sampled,
                                                 const LargeSeg* __restrict__ lsegs,
                                                 const float* __restrict__ grad,
                                                 const float* __restrict__ res, float lr,
                                                 LState* __restrict__ lstate) {
  __shared__ uint32_t s_hist[kBins0];
  __shared__ uint32_t s_wt[16];
  __shared__ uint32_t s_sel[2];
  const int li = sampled[blockIdx.x];
  const LargeSeg ls = lsegs[li];
  const SegDesc sd = segs[ls.seg];
  if (BIG && ls.sample_big)  // uniform over the workgroup
    sample_layer<16>(ls, li, sd, grad, res, lr, lstate, s_hist, s_wt, s_sel);
  else
    sample_layer<4>(ls, li, sd, grad, res, lr, lstate, s_hist, s_wt, s_sel);
}

// ------------------------------------------------------------------ stream ---
// Non-temporal store of a wave's full, 16-byte aligned chunk.
template <int V>
__device__ __forceinline__ void store_bits_nt(float* __restrict__ r, int lane, const uint32_t (&a)[V][4]) {
#pragma unroll
  for (int j = 0; j < V; ++j) {
    u32x4 o;
    o.x = a[j][0]; o.y = a[j][1]; o.z = a[j][2]; o.w = a[j][3];
    __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(r + j * 256 + lane * 4));
  }
}

// Candidate collection of one tile inside the streaming pass (all waves of the workgroup call
// it; contains one barrier).  Every entry with key >= tau goes, in index order, into the
// tile's slots (entries beyond nslot are dropped; the count written to *cnt then exceeds nslot
// and marks the tile as overflowed), and collected entries with key >= tau_hi are replaced by
// zero in `a`.  FULL: the wave's chunk is complete, no bounds checks.
template <int NW, int V, bool FULL>
__device__ __forceinline__ void stream_collect(uint32_t (&a)[V][4], int n_w, int lane, int w, uint32_t tau,
                                               uint32_t tau_hi, int32_t idx0, uint2* __restrict__ slot,
                                               int nslot, uint32_t* __restrict__ cnt, uint32_t* s_cnt) {
  // one ballot per element slot of the wave; bitwise & keeps the code free of branches
  uint64_t m[V][4];
#pragma unroll
  for (int j = 0; j < V; ++j) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool ge = (a[j][c] & 0x7FFFFFFFu) >= tau;
      if (FULL) m[j][c] = __builtin_amdgcn_ballot_w64(ge);
      else m[j][c] = __builtin_amdgcn_ballot_w64(ge & (j * 256 + lane * 4 + c < n_w));
    }
  }
  uint32_t wtot = 0;
#pragma unroll
  for (int j = 0; j < V; ++j)
    wtot += (uint32_t)(__popcll(m[j][0]) + __popcll(m[j][1]) + __popcll(m[j][2]) + __popcll(m[j][3]));
  if (lane == 0) s_cnt[w] = wtot;
  __syncthreads();
  uint32_t base = 0, total = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    const uint32_t t = s_cnt[i];
    if (i < w) base += t;
    total += t;
  }
  if (threadIdx.x == 0) *cnt = total;
  if (wtot == 0) return;  // wave-uniform
#pragma unroll
  for (int j = 0; j < V; ++j) {
    const uint32_t tot =
        (uint32_t)(__popcll(m[j][0]) + __popcll(m[j][1]) + __popcll(m[j][2]) + __popcll(m[j][3]));
    if (tot) {  // wave-uniform
      const int e = j * 256 + lane * 4;
      // slot of the lane's first candidate of this round, then one predicated store and one
      // select per component
      uint32_t pos = base + mbcnt64(m[j][0]) + mbcnt64(m[j][1]) + mbcnt64(m[j][2]) + mbcnt64(m[j][3]);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t key = a[j][c] & 0x7FFFFFFFu;
        const bool f = FULL ? key >= tau : ((key >= tau) & (e + c < n_w));
        const bool put = f & (pos < (uint32_t)nslot);
        if (put) slot[pos] = make_uint2((uint32_t)(idx0 + e + c), a[j][c]);
        // an entry at or above tau_hi is expected to be kept: its residual is written as zero
        // right here (its value is safe in the slot); the final pass corrects the few entries
        // for which that expectation turns out wrong
        a[j][c] = (put & (key >= tau_hi)) ? 0u : a[j][c];
        pos += f ? 1u : 0u;
      }
      base += tot;
    }
  }
}

// The one pass over grad and residual of every large layer: acc = residual + lr*grad is
// written into the residual buffer (it is the final residual everywhere but at the k kept
// entries).  Tiles of sampled layers also collect, in index order, the entries with
// key >= tau into the tile's slots, and write zero instead of acc for the collected entries
// with key >= tau_hi (the sample's estimate of the k-th largest key: most of them are kept, so
// most kept entries get their zero in this pass instead of a scattered write later); tiles of
// the other layers add to the layer's histogram of key bits 30..20.  Both arrays are touched
// exactly once, so full aligned tiles use non-temporal 16-byte loads and stores.  The launch
// adds kStreamLdsPad bytes of unused dynamic LDS per workgroup to cap the workgroups per CU.
template <int NW, int V>
__global__ __launch_bounds__(NW * 64) void k_stream(const TileDesc* __restrict__ tiles,
                                                const float* __restrict__ grad,
                                                float* __restrict__ res, float lr,
                                                const LState* __restrict__ lstate,
                                                uint32_t* __restrict__ chunk_cnt,
                                                uint2* __restrict__ slots, int nslot,
                                                uint32_t* __restrict__ ghist) {
  __shared__ uint32_t s_hist[kBins0];
  __shared__ uint32_t s_cnt[NW];
  static_assert(NW * V * 256 == kTile, "the workgroup covers exactly one tile");
  constexpr int NT = NW * 64, WC = V * 256;  // threads per workgroup, elements per wave
  const TileDesc td = tiles[blockIdx.x];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const bool collect = td.ctile >= 0;  // uniform over the workgroup
  uint32_t tau = 0, tau_hi = 0xFFFFFFFFu;
  if (collect) {
    tau = lstate[td.seg].tau;
    tau_hi = lstate[td.seg].tau_hi;
  } else {
    for (int i = tid; i < kBins0; i += NT) s_hist[i] = 0u;
  }
  const float* g = grad + td.start + w * WC;
  float* r = res + td.start + w * WC;
  const int n_w = td.n - w * WC;
  const bool vec = aligned16(g, r);
  uint32_t a[V][4];
  const bool fast = vec && td.n == kTile;  // uniform over the workgroup
  if (fast) {
    f32x4 gv[V], rv[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const int e = j * 256 + lane * 4;
      gv[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g + e));
      rv[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(r + e));
    }
#pragma unroll
    for (int j = 0; j < V; ++j) {
      a[j][0] = acc_bits(gv[j].x, rv[j].x, lr);
      a[j][1] = acc_bits(gv[j].y, rv[j].y, lr);
      a[j][2] = acc_bits(gv[j].z, rv[j].z, lr);
      a[j][3] = acc_bits(gv[j].w, rv[j].w, lr);
    }
  } else {
    load_acc<V>(g, r, n_w, lr, vec, lane, a);
  }
  if (collect) {
    uint2* slot = slots + (int64_t)td.ctile * nslot;
    uint32_t* cnt = chunk_cnt + td.ctile;
    const int32_t idx0 = td.local0 + w * WC;
    if (fast) stream_collect<NW, V, true>(a, n_w, lane, w, tau, tau_hi, idx0, slot, nslot, cnt, s_cnt);
    else stream_collect<NW, V, false>(a, n_w, lane, w, tau, tau_hi, idx0, slot, nslot, cnt, s_cnt);
    if (fast) store_bits_nt<V>(r, lane, a);
    else store_bits<V>(r, n_w, vec, lane, a);
  } else {
    if (fast) store_bits_nt<V>(r, lane, a);
    else store_bits<V>(r, n_w, vec, lane, a);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < V; ++j) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int e = j * 256 + lane * 4 + c;
        hist_add_peeled(s_hist, e < n_w ? (a[j][c] & 0x7FFFFFFFu) >> 20 : 0xFFFFFFFFu, lane);
      }
    }
    __syncthreads();
    uint32_t* gh = ghist + (int64_t)td.seg * kHistStride;
    for (int i = tid; i < kBins0; i += NT) {
      const uint32_t h = s_hist[i];
      if (h) atomicAdd(&gh[i], h);
    }
  }
}

// Per large layer: exclusive scan of the chunks' candidate counts, the verdict on the
// guess (MODE_SPARSE iff no chunk overflowed, at least k candidates, list fits), and, for
// layers in MODE_DENSE, their tiles appended to the work list of the fallback kernels.
__global__ __launch_bounds__(1024) void k_cscan(const SegDesc* __restrict__ segs,
                                                const LargeSeg* __restrict__ lsegs,
                                                LState* __restrict__ lstate,
                                                const uint32_t* __restrict__ chunk_cnt, int nslot,
                                                uint32_t* __restrict__ chunk_off,
                                                uint32_t* __restrict__ counter,
                                                int32_t* __restrict__ items) {
  __shared__ uint32_t s_wt[16];
  __shared__ uint32_t s_base;
  const int li = blockIdx.x;
  const LargeSeg ls = lsegs[li];
  const int tid = threadIdx.x;
  uint32_t mode = MODE_DENSE;
  if (ls.cand_class != CAND_NONE) {  // uniform over the workgroup
    uint32_t carry = 0;
    int over = 0;
    for (int base = ls.chunk_begin; base < ls.chunk_end; base += 8192) {
      const int i0 = base + tid * 8;
      uint32_t v[8], s = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        v[e] = (i0 + e < ls.chunk_end) ? chunk_cnt[i0 + e] : 0u;
        over |= v[e] > (uint32_t)nslot;
        s += v[e];
      }
      uint32_t tot;
      const uint32_t incl = block_incl_scan<1024>(s, s_wt, tot);
      uint32_t run = carry + incl - s;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (i0 + e < ls.chunk_end) chunk_off[i0 + e] = run;
        run += v[e];
      }
      carry += tot;
    }
    over = __syncthreads_or(over);
    const uint32_t k = (uint32_t)segs[ls.seg].k;
    if (!over && carry >= k && carry <= (uint32_t)ls.cap) mode = MODE_SPARSE;
    if (tid == 0) lstate[li].ncand = carry;
  }
  if (tid == 0) lstate[li].mode = mode;
  if (mode == MODE_DENSE) {
    const int nt = ls.tile_end - ls.tile_begin;
    if (tid == 0) s_base = atomicAdd(counter, (uint32_t)nt);
    __syncthreads();
    const uint32_t b = s_base;
    for (int j = tid; j < nt; j += 1024) items[b + j] = ls.tile_begin + j;
  }
}

// Copy the tiles' slots into the layer's contiguous candidate list (index order is kept
// because tiles are laid out in index order); for layers whose guess was rejected, undo the
// streaming pass's early zeros instead.  A wave takes 64 consecutive tiles; lane l
// learns tile l's count and destination, then the wave copies all their entries 64 at a
// time: for the e-th entry the owning tile is found by a binary search over the lanes'
// exclusive counts (shuffles), so neighbouring lanes read neighbouring slots of one tile
// and write neighbouring list positions.
__global__ __launch_bounds__(256) void k_cgather(int n_chunks, const int32_t* __restrict__ chunk_lseg,
                                                 const LargeSeg* __restrict__ lsegs,
                                                 const LState* __restrict__ lstate,
                                                 const uint32_t* __restrict__ chunk_cnt,
                                                 const uint32_t* __restrict__ chunk_off,
                                                 const uint2* __restrict__ slots, int nslot,
                                                 uint2* __restrict__ cand,
                                                 const SegDesc* __restrict__ segs,
                                                 float* __restrict__ res) {
  const int lane = lane_id();
  const int c0 = (int)((blockIdx.x * 256u + threadIdx.x) >> 6) * 64;  // first tile of the wave
  if (c0 >= n_chunks) return;  // wave-uniform
  const int c = c0 + lane;
  uint32_t cnt = 0;
  int64_t dst = 0;
  if (c < n_chunks) {
    const int li = chunk_lseg[c];
    const LState st = lstate[li];
    if (st.mode == MODE_SPARSE) {
      cnt = chunk_cnt[c];
      dst = lsegs[li].cand_base + chunk_off[c];
    } else {
      // the layer falls back to the multi-pass route, which reads acc from the residual
      // buffer: give the entries that the streaming pass zeroed (slotted, key >= tau_hi)
      // their acc back.  Rare path, one lane per tile.
      const uint32_t stored = chunk_cnt[c] < (uint32_t)nslot ? chunk_cnt[c] : (uint32_t)nslot;
      float* rl = res + segs[lsegs[li].seg].offset;
      const uint2* src = slots + (int64_t)c * nslot;
      for (uint32_t q = 0; q < stored; ++q) {
        const uint2 en = src[q];
        if ((en.y & 0x7FFFFFFFu) >= st.tau_hi) rl[en.x] = __uint_as_float(en.y);
      }
    }
  }
  const uint32_t incl = wave_incl_scan(cnt, lane);
  const uint32_t pre = incl - cnt;
  const uint32_t total = __shfl(incl, 63, 64);
  const uint32_t dst_lo = (uint32_t)dst, dst_hi = (uint32_t)(dst >> 32);
  for (uint32_t base = 0; base < total; base += 64) {  // wave-uniform trip count
    const bool live = base + lane < total;
    const uint32_t e = live ? base + lane : total - 1;  // idle lanes search along, then skip the copy
    int lo = 0, hi = 63;  // last lane whose exclusive count is <= e: the tile that owns entry e
#pragma unroll
    for (int step = 0; step < 6; ++step) {
      const int mid = (lo + hi + 1) >> 1;
      const uint32_t v = __shfl(pre, mid, 64);
      if (v <= e) lo = mid; else hi = mid - 1;
    }
    const uint32_t p0 = __shfl(pre, lo, 64);
    const uint32_t d_lo = __shfl(dst_lo, lo, 64), d_hi = __shfl(dst_hi, lo, 64);
    if (live) {
      const uint32_t q = e - p0;
      const int64_t d = (int64_t)(((uint64_t)d_hi << 32) | d_lo) + q;
      cand[d] = slots[(int64_t)(c0 + lo) * nslot + q];
    }
  }
}

// ------------------------------------------------------------------ multi-block select
// The same radix-select passes serve two sources: CAND = false walks the acc values in
// the residual buffer (fallback; tiles come from the device-built work list `items`),
// CAND = true walks a layer's candidate list (tiles of kTile list entries).
struct TileWork {
  float* res;          // dense: the tile's residual data
  const uint2* cand;   // candidate source: the tile's list entries
  int n;               // valid entries
  int lseg;
  int local0;          // dense: layer-local index of the first element
  int slot;            // index into tile_gt / tile_eq
  bool active;         // candidate source: the layer is in MODE_SPARSE
  bool skip_level0;    // dense: level-0 histogram already made by the streaming pass
};

// Returns true if the tile has entries to process.
template <bool CAND>
__device__ __forceinline__ bool get_tile(int item, const TileDesc* __restrict__ tiles,
                                         const int32_t* __restrict__ items, float* res,
                                         const uint2* cand, const LState* __restrict__ lstate, int n_tiles,
                                         TileWork& tw) {
  if (CAND) {
    const TileDesc td = tiles[item];
    const LState st = lstate[td.seg];
    tw.lseg = td.seg;
    tw.slot = n_tiles + item;
    tw.local0 = td.local0;
    tw.res = nullptr;
    tw.cand = cand + td.start;
    tw.skip_level0 = false;
    tw.active = st.mode == MODE_SPARSE;
    const int left = (int)st.ncand - td.local0;
    tw.n = left < td.n ? left : td.n;
    return tw.active && tw.n > 0;
  } else {
    const int t = items[item];
    const TileDesc td = tiles[t];
    tw.lseg = td.seg;
    tw.slot = t;
    tw.local0 = td.local0;
    tw.res = res + td.start;
    tw.cand = nullptr;
    tw.n = td.n;
    tw.active = true;
    tw.skip_level0 = td.ctile < 0;
    return true;
  }
}

template <bool CAND>
__device__ __forceinline__ void load_tile(const TileWork& tw, int w, int lane, uint32_t (&a)[kTileV][4]) {
  const int n_w = tw.n - w * kWaveChunk;
  if (CAND) {
    load_cand_bits<kTileV>(tw.cand + w * kWaveChunk, n_w, lane, a);
  } else {
    const float* r = tw.res + w * kWaveChunk;
    load_bits<kTileV>(r, n_w, aligned16(r, r), lane, a);
  }
}

// The three per-tile kernels below serve both sources in one launch: workgroups
// [0, n_cblocks) take one candidate tile each (ctiles[blockIdx.x]); the kDenseGrid workgroups
// after them walk the fallback work list (items[0 .. *counter)), which is empty unless a
// layer's guess was rejected.

// One digit of the radix select, decided from the layer's histogram of that digit (complete
// since the previous launch): every workgroup that needs the result computes it for itself,
// and the workgroup that holds the layer's first tile also records it in the layer's state for
// the launches after this one.  k_before: entries still to take before this digit.
// Returns false if the histogram holds fewer than k_before entries (nothing to select).
__device__ __forceinline__ bool decide_digit(const uint32_t* __restrict__ gh, int nb, int shift, uint32_t p_before,
                                             uint32_t k_before, uint32_t* s_wt, uint32_t* s_sel,
                                             uint32_t& p_after, uint32_t& k_after) {
  __syncthreads();
  if (threadIdx.x == 0) { s_sel[0] = 0u; s_sel[1] = 0u; }
  __syncthreads();
  block_find_bucket<256>(gh, nb, k_before, s_wt, s_sel);
  p_after = p_before | (s_sel[0] << shift);
  k_after = s_sel[1];
  return k_after != 0u;
}

// Histogram of one radix digit over the entries whose higher key bits equal the prefix
// (levels 1 and 2 first decide the digit before theirs from its histogram).
template <int LEVEL, bool CAND>
__device__ __forceinline__ void hist_tiles(int first, int end, int step, uint32_t* s_hist, uint32_t* s_wt,
                                           uint32_t* s_sel, const TileDesc* __restrict__ tiles,
                                           const int32_t* __restrict__ items, int n_tiles,
                                           const LargeSeg* __restrict__ lsegs, const SegDesc* __restrict__ segs,
                                           float* __restrict__ res, const uint2* __restrict__ cand,
                                           LState* __restrict__ lstate, uint32_t* __restrict__ ghist) {
  constexpr int shift = LEVEL == 0 ? 20 : (LEVEL == 1 ? 10 : 0);
  constexpr uint32_t mask = LEVEL == 0 ? 0u : (LEVEL == 1 ? 0x7FF00000u : 0x7FFFFC00u);
  constexpr int nb = LEVEL == 0 ? kBins0 : kBins12;
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  for (int item = first; item < end; item += step) {
    TileWork tw;
    if (!get_tile<CAND>(item, tiles, items, res, cand, lstate, n_tiles, tw)) continue;
    if (LEVEL == 0 && tw.skip_level0) continue;
    uint32_t* gh = ghist + (int64_t)tw.lseg * kHistStride;
    uint32_t prefix = 0u;
    if (LEVEL == 1) {
      uint32_t kr;
      if (!decide_digit(gh, kBins0, 20, 0u, (uint32_t)segs[lsegs[tw.lseg].seg].k, s_wt, s_sel, prefix, kr)) continue;
      if (tw.local0 == 0 && tid == 0) { lstate[tw.lseg].p0 = prefix; lstate[tw.lseg].k0 = kr; }
    } else if (LEVEL == 2) {
      uint32_t kr;
      const uint32_t p0 = lstate[tw.lseg].p0, k0 = lstate[tw.lseg].k0;
      if (!decide_digit(gh + kHistLevel1, kBins12, 10, p0, k0, s_wt, s_sel, prefix, kr)) continue;
      if (tw.local0 == 0 && tid == 0) { lstate[tw.lseg].p1 = prefix; lstate[tw.lseg].k1 = kr; }
    }
    __syncthreads();
    for (int i = tid; i < nb; i += 256) s_hist[i] = 0u;
    uint32_t a[kTileV][4];
    load_tile<CAND>(tw, w, lane, a);
    const int n_w = tw.n - w * kWaveChunk;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kTileV; ++j) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int e = j * 256 + lane * 4 + c;
        const uint32_t key = a[j][c] & 0x7FFFFFFFu;
        const bool in = e < n_w && (key & mask) == prefix;
        if (LEVEL == 0) hist_add_peeled(s_hist, in ? key >> shift : 0xFFFFFFFFu, lane);
        else if (in) atomicAdd(&s_hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
      }
    }
    __syncthreads();
    uint32_t* gl = gh + (LEVEL == 0 ? 0 : (LEVEL == 1 ? kHistLevel1 : kHistLevel2));
    for (int i = tid; i < nb; i += 256) {
      const uint32_t h = s_hist[i];
      if (h) atomicAdd(&gl[i], h);
    }
  }
}

template <int LEVEL>
__global__ __launch_bounds__(256) void k_hist(int n_cblocks, const TileDesc* __restrict__ ctiles,
                                              const TileDesc* __restrict__ tiles,
                                              const int32_t* __restrict__ items,
                                              const uint32_t* __restrict__ counter, int n_tiles,
                                              const LargeSeg* __restrict__ lsegs,
                                              const SegDesc* __restrict__ segs,
                                              float* __restrict__ res,
                                              const uint2* __restrict__ cand,
                                              LState* __restrict__ lstate,
                                              uint32_t* __restrict__ ghist) {
  __shared__ uint32_t s_hist[LEVEL == 0 ? kBins0 : kBins12];
  __shared__ uint32_t s_wt[4];
  __shared__ uint32_t s_sel[2];
  const int b = (int)blockIdx.x;
  if (b < n_cblocks)  // uniform over the workgroup
    hist_tiles<LEVEL, true>(b, b + 1, 1, s_hist, s_wt, s_sel, ctiles, items, n_tiles, lsegs, segs, res, cand, lstate,
                            ghist);
  else
    hist_tiles<LEVEL, false>(b - n_cblocks, (int)*counter, kDenseGrid, s_hist, s_wt, s_sel, tiles, items, n_tiles,
                             lsegs, segs, res, cand, lstate, ghist);
}

// Decides the last digit (which fixes the k-th largest key T and the number of entries equal
// to T to take), then counts per tile how many keys are above T and how many equal T.
template <bool CAND>
__device__ __forceinline__ void count_tiles(int first, int end, int step, uint32_t* s_g, uint32_t* s_e,
                                            uint32_t* s_wt, uint32_t* s_sel,
                                            const TileDesc* __restrict__ tiles,
                                            const int32_t* __restrict__ items, int n_tiles,
                                            float* __restrict__ res, const uint2* __restrict__ cand,
                                            LState* __restrict__ lstate, const uint32_t* __restrict__ ghist,
                                            uint32_t* __restrict__ tile_gt,
                                            uint32_t* __restrict__ tile_eq) {
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  for (int item = first; item < end; item += step) {
    TileWork tw;
    if (!get_tile<CAND>(item, tiles, items, res, cand, lstate, n_tiles, tw)) {
      // an empty candidate tile of a layer in candidate mode still takes part in the scan
      if (CAND && tw.active && tid == 0) { tile_gt[tw.slot] = 0u; tile_eq[tw.slot] = 0u; }
      continue;
    }
    uint32_t T, rtake;
    const uint32_t p1 = lstate[tw.lseg].p1, k1 = lstate[tw.lseg].k1;
    if (!decide_digit(ghist + (int64_t)tw.lseg * kHistStride + kHistLevel2, kBins12, 0, p1, k1, s_wt, s_sel, T,
                      rtake))
      continue;
    if (tw.local0 == 0 && tid == 0) { lstate[tw.lseg].prefix = T; lstate[tw.lseg].k_rem = rtake; }
    uint32_t a[kTileV][4];
    load_tile<CAND>(tw, w, lane, a);
    uint32_t cg, ce;
    lane_count<kTileV>(a, tw.n - w * kWaveChunk, lane, T, cg, ce);
    cg = wave_sum(cg);
    ce = wave_sum(ce);
    __syncthreads();
    if (lane == 0) { s_g[w] = cg; s_e[w] = ce; }
    __syncthreads();
    if (tid == 0) {
      tile_gt[tw.slot] = s_g[0] + s_g[1] + s_g[2] + s_g[3];
      tile_eq[tw.slot] = s_e[0] + s_e[1] + s_e[2] + s_e[3];
    }
  }
}

__global__ __launch_bounds__(256) void k_count(int n_cblocks, const TileDesc* __restrict__ ctiles,
                                               const TileDesc* __restrict__ tiles,
                                               const int32_t* __restrict__ items,
                                               const uint32_t* __restrict__ counter, int n_tiles,
                                               float* __restrict__ res,
                                               const uint2* __restrict__ cand,
                                               LState* __restrict__ lstate,
                                               const uint32_t* __restrict__ ghist,
                                               uint32_t* __restrict__ tile_gt,
                                               uint32_t* __restrict__ tile_eq) {
  __shared__ uint32_t s_g[4], s_e[4];
  __shared__ uint32_t s_wt[4];
  __shared__ uint32_t s_sel[2];
  const int b = (int)blockIdx.x;
  if (b < n_cblocks)  // uniform over the workgroup
    count_tiles<true>(b, b + 1, 1, s_g, s_e, s_wt, s_sel, ctiles, items, n_tiles, res, cand, lstate, ghist, tile_gt,
                      tile_eq);
  else
    count_tiles<false>(b - n_cblocks, (int)*counter, kDenseGrid, s_g, s_e, s_wt, s_sel, tiles, items, n_tiles, res,
                       cand, lstate, ghist, tile_gt, tile_eq);
}

// Exclusive scan of the per-tile counts inside each large layer (in place): over the
// layer's dense tiles in MODE_DENSE, over its candidate tiles in MODE_SPARSE.
__global__ __launch_bounds__(1024) void k_scan(const LargeSeg* __restrict__ lsegs,
                                               const LState* __restrict__ lstate, int n_tiles,
                                               uint32_t* __restrict__ tile_gt,
                                               uint32_t* __restrict__ tile_eq) {
  __shared__ uint32_t s_wt[16];
  const LargeSeg ls = lsegs[blockIdx.x];
  const uint32_t mode = lstate[blockIdx.x].mode;
  int begin, end;
  if (mode == MODE_DENSE) { begin = ls.tile_begin; end = ls.tile_end; }
  else if (ls.cand_class == CAND_LARGE) { begin = n_tiles + ls.ctile_begin; end = n_tiles + ls.ctile_end; }
  else return;
  uint32_t carry_g = 0, carry_e = 0;
  for (int base = begin; base < end; base += 1024) {
    const int i = base + threadIdx.x;
    const uint32_t vg = i < end ? tile_gt[i] : 0u;
    const uint32_t ve = i < end ? tile_eq[i] : 0u;
    uint32_t tg, te;
    const uint32_t ig = block_incl_scan<1024>(vg, s_wt, tg);
    const uint32_t ie = block_incl_scan<1024>(ve, s_wt, te);
    if (i < end) {
      tile_gt[i] = carry_g + ig - vg;
      tile_eq[i] = carry_e + ie - ve;
    }
    carry_g += tg;
    carry_e += te;
  }
}

// Final pass: ordered emission of the kept pairs and zeroing of their residual slots.
template <bool CAND>
__device__ __forceinline__ void emit_tiles(int first, int end, int step, uint32_t* s_g, uint32_t* s_e,
                                           const TileDesc* __restrict__ tiles,
                                           const int32_t* __restrict__ items, int n_tiles,
                                           const LargeSeg* __restrict__ lsegs,
                                           const SegDesc* __restrict__ segs, float* __restrict__ res,
                                           const uint2* __restrict__ cand,
                                           const LState* __restrict__ lstate,
                                           const uint32_t* __restrict__ tile_gt,
                                           const uint32_t* __restrict__ tile_eq,
                                           int32_t* __restrict__ out_idx, float* __restrict__ out_val) {
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  for (int item = first; item < end; item += step) {
    TileWork tw;
    if (!get_tile<CAND>(item, tiles, items, res, cand, lstate, n_tiles, tw)) continue;
    const LState st = lstate[tw.lseg];
    const uint32_t T = st.prefix, rtake = st.k_rem;
    const uint32_t tg = tile_gt[tw.slot], te = tile_eq[tw.slot];
    const SegDesc sd = segs[lsegs[tw.lseg].seg];
    const int n_w = tw.n - w * kWaveChunk;
    uint32_t a[kTileV][4];
    load_tile<CAND>(tw, w, lane, a);
    uint32_t cg, ce;
    lane_count<kTileV>(a, n_w, lane, T, cg, ce);
    cg = wave_sum(cg);
    ce = wave_sum(ce);
    __syncthreads();
    if (lane == 0) { s_g[w] = cg; s_e[w] = ce; }
    __syncthreads();
    uint32_t gb = tg, eb = te;
    for (int i = 0; i < w; ++i) { gb += s_g[i]; eb += s_e[i]; }
    if (CAND) {
      // every wave runs: entries zeroed by the streaming pass but not kept must get acc back
      wave_emit<kTileV, EMIT_CAND>(a, n_w, lane, T, rtake, gb, eb, (uint32_t)sd.k, 0, out_idx + sd.out_offset,
                                   out_val + sd.out_offset, res + sd.offset, false, tw.cand + w * kWaveChunk,
                                   st.tau_hi);
    } else {
      // nothing to emit in this wave if it holds no key above T and its ties come too late
      if (cg == 0 && (ce == 0 || eb >= rtake)) continue;
      float* r = tw.res + w * kWaveChunk;
      wave_emit<kTileV, EMIT_ZERO>(a, n_w, lane, T, rtake, gb, eb, (uint32_t)sd.k, tw.local0 + w * kWaveChunk,
                                   out_idx + sd.out_offset, out_val + sd.out_offset, r, aligned16(r, r), nullptr,
                                   0u);
    }
  }
}

__global__ __launch_bounds__(256) void k_emit(int n_cblocks, const TileDesc* __restrict__ ctiles,
                                              const TileDesc* __restrict__ tiles,
                                              const int32_t* __restrict__ items,
                                              const uint32_t* __restrict__ counter, int n_tiles,
                                              const LargeSeg* __restrict__ lsegs,
                                              const SegDesc* __restrict__ segs,
                                              float* __restrict__ res,
                                              const uint2* __restrict__ cand,
                                              const LState* __restrict__ lstate,
                                              const uint32_t* __restrict__ tile_gt,
                                              const uint32_t* __restrict__ tile_eq,
                                              int32_t* __restrict__ out_idx,
                                              float* __restrict__ out_val) {
  __shared__ uint32_t s_g[4], s_e[4];
  const int b = (int)blockIdx.x;
  if (b < n_cblocks)  // uniform over the workgroup
    emit_tiles<true>(b, b + 1, 1, s_g, s_e, ctiles, items, n_tiles, lsegs, segs, res, cand, lstate,
                     tile_gt, tile_eq, out_idx, out_val);
  else
    emit_tiles<false>(b - n_cblocks, (int)*counter, kDenseGrid, s_g, s_e, tiles, items, n_tiles, lsegs, segs, res,
                      cand, lstate, tile_gt, tile_eq, out_idx, out_val);
}

// ------------------------------------------------------------------ merge ----
// Algorithm 1 lines 8-9.  Two kernels.
//
// k_merge_bounds: for every worker and layer, where each 8192-element tile of the dense
// update starts in the worker's sorted index list: bounds[p][slot0 + t] = first list position
// whose index lies in tile t or later; bounds[p][slot0 + ntiles] = k.  One pass over the lists.
__global__ __launch_bounds__(256) void k_merge_bounds(const BChunk* __restrict__ chunks,
                                                      const SegDesc* __restrict__ segs,
                                                      const int32_t* __restrict__ idx, int64_t stride_k,
                                                      int nb, int32_t* __restrict__ bounds) {
  const BChunk bc = chunks[blockIdx.x];
  const int p = blockIdx.y;
  const SegDesc sd = segs[bc.seg];
  const int32_t* li = idx + (int64_t)p * stride_k + sd.out_offset;
  int32_t* b = bounds + (int64_t)p * nb + bc.slot0;
  const int jend = sd.k < bc.j0 + kBoundChunk ? sd.k : bc.j0 + kBoundChunk;
  for (int j = bc.j0 + (int)threadIdx.x; j < jend; j += 256) {
    // indices are clamped into the layer so that bad input cannot write outside the row
    int i1 = li[j];
    i1 = i1 < 0 ? 0 : (i1 >= sd.d ? sd.d - 1 : i1);
    const int t = i1 / kMergeTile;
    int tp = -1;
    if (j > 0) {
      int i0 = li[j - 1];
      i0 = i0 < 0 ? 0 : (i0 >= sd.d ? sd.d - 1 : i0);
      tp = i0 / kMergeTile;
    }
    for (int q = tp + 1; q <= t; ++q) b[q] = j;
    if (j == sd.k - 1)
      for (int q = t + 1; q <= bc.ntiles; ++q) b[q] = sd.k;
  }
}

// Accumulation shared by the merge-type kernels: the workgroup that owns one tile of the
// dense layout loads the entries of all workers that fall into the tile (found through the
// bounds, no searching) and adds them into the LDS tile s_acc in worker order (one barrier per
// worker; inside one worker the indices are distinct).  T = float: binary32 adds, the sum the
// method defines.  T = double: exact-order double sums for the delta metric.
// Returns the number of entries that fell into the tile.
template <typename T>
__device__ __forceinline__ uint32_t merge_accumulate(T* s_acc, uint32_t* s_start, int32_t* s_lo, uint32_t* s_wt,
                                                     const TileDesc& td, const SegDesc& sd, int slot,
                                                     const int32_t* __restrict__ idx,
                                                     const float* __restrict__ val, int P, int64_t stride_k,
                                                     int nb, const int32_t* __restrict__ bounds) {
  const int tid = threadIdx.x;
  uint32_t entries = 0;
  for (int i = tid; i < kMergeTile; i += 256) s_acc[i] = (T)0;
  for (int p0 = 0; p0 < P; p0 += 256) {
    const int np = P - p0 < 256 ? P - p0 : 256;
    int lo = 0;
    uint32_t cnt = 0;
    if (tid < np) {
      const int32_t* b = bounds + (int64_t)(p0 + tid) * nb + slot;
      int hi = b[1];
      lo = b[0];
      lo = lo < 0 ? 0 : (lo > sd.k ? sd.k : lo);
      hi = hi < 0 ? 0 : (hi > sd.k ? sd.k : hi);
      cnt = hi > lo ? (uint32_t)(hi - lo) : 0u;
    }
    uint32_t total;
    const uint32_t incl = block_incl_scan<256>(cnt, s_wt, total);
    s_start[tid] = incl - cnt;
    s_lo[tid] = lo;
    if (tid == 0) s_start[256] = total;
    __syncthreads();
    entries += total;
    for (uint32_t base = 0; base < total; base += 1024) {
      int pe[4];
      uint32_t off[4];
      float v[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t e = base + (uint32_t)(r * 256 + tid);
        pe[r] = -1;
        off[r] = 0xFFFFFFFFu;
        v[r] = 0.f;
        if (e < total) {
          int a = 0, z = np;  // last worker q with s_start[q] <= e (skips workers without entries here)
          while (a < z) {
            const int mid = (a + z) >> 1;
            if (s_start[mid] <= e) a = mid + 1; else z = mid;
          }
          const int q = a - 1;
          const int64_t gi = (int64_t)(p0 + q) * stride_k + sd.out_offset + s_lo[q] + (int)(e - s_start[q]);
          off[r] = (uint32_t)(idx[gi] - td.local0);
          v[r] = val[gi];
          pe[r] = q;
        }
      }
      // workers present in this pass (uniform over the workgroup)
      int qf, ql;
      {
        const uint32_t e0 = base, e1 = (base + 1024 < total ? base + 1024 : total) - 1;
        int a = 0, z = np;
        while (a < z) { const int mid = (a + z) >> 1; if (s_start[mid] <= e0) a = mid + 1; else z = mid; }
        qf = a - 1;
        a = 0; z = np;
        while (a < z) { const int mid = (a + z) >> 1; if (s_start[mid] <= e1) a = mid + 1; else z = mid; }
        ql = a - 1;
      }
      for (int q = qf; q <= ql; ++q) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (pe[r] == q && off[r] < (uint32_t)td.n) {
            if (sizeof(T) == 4) s_acc[off[r]] = (T)__fadd_rn((float)s_acc[off[r]], v[r]);
            else s_acc[off[r]] = s_acc[off[r]] + (T)v[r];
          }
        }
        __syncthreads();
      }
    }
    __syncthreads();
  }
  return entries;
}

// k_merge<false>: the dense averaged update (Algorithm 1 lines 8-9): the whole tile is written
// once, divided by P.  k_merge<true>: the parameter step of Algorithm 1 line 9 applied in
// place, v -= update, touching only the elements whose sum is not zero (v - 0 == v bit for bit,
// and a sum that starts from +0.0f is never -0.0f).  No atomics, fixed summation order.
template <bool APPLY>
__global__ __launch_bounds__(256) void k_merge(const TileDesc* __restrict__ mtiles,
                                               const SegDesc* __restrict__ segs,
                                               const int32_t* __restrict__ idx,
                                               const float* __restrict__ val, int P,
                                               int64_t stride_k, int nb,
                                               const int32_t* __restrict__ bounds,
                                               float* __restrict__ out) {
  __shared__ float s_acc[kMergeTile];
  __shared__ uint32_t s_start[257];
  __shared__ int32_t s_lo[256];
  __shared__ uint32_t s_wt[4];
  __shared__ uint32_t s_claim[APPLY ? kMergeTile / 32 : 1];
  const TileDesc td = mtiles[blockIdx.x];
  const SegDesc sd = segs[td.seg];
  const int tid = threadIdx.x;
  const int slot = (int)blockIdx.x + td.seg;  // every earlier layer owns one extra (end) slot
  if (APPLY) s_claim[tid] = 0u;  // kMergeTile / 32 = 256 words; the accumulation's barriers order this
  const uint32_t entries =
      merge_accumulate<float>(s_acc, s_start, s_lo, s_wt, td, sd, slot, idx, val, P, stride_k, nb, bounds);
  // sum / P: for P a power of two the product with 1/P is the same binary32 value as the
  // quotient (an exact scaling, rounded identically when the result is subnormal), and it is
  // much cheaper than a correctly rounded division
  const float fp = (float)P;
  const bool pow2 = (P & (P - 1)) == 0;
  const float inv = 1.0f / fp;
  float* u = out + td.start;
  if (APPLY) {
    if (entries == 0) return;  // uniform over the workgroup
    if (P <= 256) {
      // One pass of the accumulation covered all workers, so its entry table (s_start, s_lo) is
      // still valid: walk the entries again and let the first thread that claims an element's
      // bit apply the element's sum.  Touches the selected elements only, in one round trip.
      const uint32_t total = s_start[256];
      for (uint32_t base = 0; base < total; base += 256) {
        const uint32_t e = base + (uint32_t)tid;
        if (e < total) {
          int a = 0, z = P;  // last worker q with s_start[q] <= e
          while (a < z) {
            const int mid = (a + z) >> 1;
            if (s_start[mid] <= e) a = mid + 1; else z = mid;
          }
          const int q = a - 1;
          const int64_t gi = (int64_t)q * stride_k + sd.out_offset + s_lo[q] + (int)(e - s_start[q]);
          const uint32_t off = (uint32_t)(idx[gi] - td.local0);
          if (off < (uint32_t)td.n) {
            const uint32_t bit = 1u << (off & 31u);
            if (!(atomicOr(&s_claim[off >> 5], bit) & bit)) {
              const float sacc = s_acc[off];
              if (sacc != 0.0f) u[off] = __fsub_rn(u[off], pow2 ? __fmul_rn(sacc, inv) : __fdiv_rn(sacc, fp));
            }
          }
        }
      }
      return;
    }
    for (int e = tid; e < td.n; e += 256) {
      const float sacc = s_acc[e];
      if (sacc != 0.0f) u[e] = __fsub_rn(u[e], pow2 ? __fmul_rn(sacc, inv) : __fdiv_rn(sacc, fp));
    }
    return;
  }
  const bool vec = aligned16(u, u);
  for (int e = tid * 4; e < td.n; e += 1024) {
    if (vec && e + 3 < td.n) {
      const float4 sv = *reinterpret_cast<const float4*>(&s_acc[e]);
      float4 v;
      if (pow2) {
        v.x = __fmul_rn(sv.x, inv); v.y = __fmul_rn(sv.y, inv);
        v.z = __fmul_rn(sv.z, inv); v.w = __fmul_rn(sv.w, inv);
      } else {
        v.x = __fdiv_rn(sv.x, fp); v.y = __fdiv_rn(sv.y, fp);
        v.z = __fdiv_rn(sv.z, fp); v.w = __fdiv_rn(sv.w, fp);
      }
      // the update is written once and not read again by this library: non-temporal stores
      // (measured: 0.138 ms instead of 0.176 ms for 553 MB)
      f32x4 o;
      o.x = v.x; o.y = v.y; o.z = v.z; o.w = v.w;
      __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(u + e));
    } else {
      for (int c = 0; c < 4; ++c)
        if (e + c < td.n) u[e + c] = pow2 ? __fmul_rn(s_acc[e + c], inv) : __fdiv_rn(s_acc[e + c], fp);
    }
  }
}

// Section 6.2, per tile: with s = sum_p residual_p (the residuals after sparsification) and
// x = s + sum_p selected_p, the tile's parts of ||s||^2 and ||x||^2 in double.  Sums over
// workers run in worker order; the tile's two partial sums go to partials[2*tile], [2*tile+1].
__global__ __launch_bounds__(256) void k_delta_tiles(const TileDesc* __restrict__ mtiles,
                                                     const SegDesc* __restrict__ segs,
                                                     const float* __restrict__ res, int64_t res_stride,
                                                     const int32_t* __restrict__ idx,
                                                     const float* __restrict__ val, int P,
                                                     int64_t stride_k, int nb,
                                                     const int32_t* __restrict__ bounds,
                                                     double* __restrict__ partials) {
  __shared__ double s_acc[kMergeTile];
  __shared__ uint32_t s_start[257];
  __shared__ int32_t s_lo[256];
  __shared__ uint32_t s_wt[4];
  __shared__ double s_red[8];
  const TileDesc td = mtiles[blockIdx.x];
  const SegDesc sd = segs[td.seg];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const int slot = (int)blockIdx.x + td.seg;
  (void)merge_accumulate<double>(s_acc, s_start, s_lo, s_wt, td, sd, slot, idx, val, P, stride_k, nb, bounds);
  double num = 0.0, sq = 0.0;
  const float* rt = res + td.start;
  const bool vec = aligned16(rt, rt) && (res_stride & 3) == 0;
  for (int e = tid * 4; e < td.n; e += 1024) {
    double ssum[4] = {0.0, 0.0, 0.0, 0.0};
    if (vec && e + 3 < td.n) {
      const float* r = rt + e;
      // the residuals are read once: non-temporal loads, 16 workers' loads in flight per thread
      // (measured 6.75 TB/s against 6.05 TB/s with plain loads unrolled by 8)
#pragma unroll 16
      for (int p = 0; p < P; ++p) {
        const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(r + (int64_t)p * res_stride));
        ssum[0] += (double)v.x;
        ssum[1] += (double)v.y;
        ssum[2] += (double)v.z;
        ssum[3] += (double)v.w;
      }
    } else {
      for (int c = 0; c < 4; ++c)
        if (e + c < td.n)
          for (int p = 0; p < P; ++p) ssum[c] += (double)rt[e + c + (int64_t)p * res_stride];
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (e + c < td.n) {
        const double x = ssum[c] + s_acc[e + c];
        num += ssum[c] * ssum[c];
        sq += x * x;
      }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    num += __shfl_xor(num, o, 64);
    sq += __shfl_xor(sq, o, 64);
  }
  if (lane == 0) { s_red[w] = num; s_red[4 + w] = sq; }
  __syncthreads();
  if (tid == 0) {
    partials[2 * (int64_t)blockIdx.x + 0] = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
    partials[2 * (int64_t)blockIdx.x + 1] = (s_red[4] + s_red[5]) + (s_red[6] + s_red[7]);
  }
}

// Section 6.2, per layer: add the tiles' partial sums in a fixed order and form
// delta = ||s||^2 / ((1 - k/d) ||x||^2)  (NaN when the denominator is 0).
// out3[3*l] = ||s||^2, out3[3*l+1] = ||x||^2, out3[3*l+2] = delta.
__global__ __launch_bounds__(256) void k_delta_finish(const SegDesc* __restrict__ segs,
                                                      const int32_t* __restrict__ seg_mtile0,
                                                      const double* __restrict__ partials,
                                                      double* __restrict__ out3) {
  __shared__ double s_a[256], s_b[256];
  const int l = blockIdx.x, tid = threadIdx.x;
  const int t0 = seg_mtile0[l], t1 = seg_mtile0[l + 1];
  double a = 0.0, b = 0.0;
  for (int t = t0 + tid; t < t1; t += 256) { a += partials[2 * (int64_t)t]; b += partials[2 * (int64_t)t + 1]; }
  s_a[tid] = a;
  s_b[tid] = b;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) { s_a[tid] += s_a[tid + o]; s_b[tid] += s_b[tid + o]; }
    __syncthreads();
  }
  if (tid == 0) {
    const SegDesc sd = segs[l];
    const double den = (1.0 - (double)sd.k / (double)sd.d) * s_b[0];
    out3[3 * l + 0] = s_a[0];
    out3[3 * l + 1] = s_b[0];
    out3[3 * l + 2] = den > 0.0 ? s_a[0] / den : __longlong_as_double(0x7FF8000000000000LL);
  }
}

// ------------------------------------------------------------------ launch ---
const char* kernel_name(int id) {
  static const char* names[K_NUM] = {
      "k_zero_u32", "k_small<4,1>", "k_small<4,8>", "k_small<16,10>", "k_sample", "k_stream", "k_cscan",
      "k_cgather", "k_small<4,1,cand>", "k_small<4,8,cand>", "k_small<16,10,cand>", "k_hist", "k_count",
      "k_scan", "k_emit", "k_merge_bounds", "k_merge", "k_merge<apply>", "k_delta_tiles", "k_delta_finish",
      "sparsify_call"};
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
  const LargeSeg* nl = nullptr;
  const LState* ns = nullptr;
  const uint2* nc = nullptr;
  if (cls == 0)
    hipLaunchKernelGGL((k_small<4, 1, false>), dim3(nseg), dim3(256), 0, s, segs, list, nl, ns, nc, grad, res, lr,
                       out_idx, out_val);
  else if (cls == 1)
    hipLaunchKernelGGL((k_small<4, 8, false>), dim3(nseg), dim3(256), 0, s, segs, list, nl, ns, nc, grad, res, lr,
                       out_idx, out_val);
  else
    hipLaunchKernelGGL((k_small<16, 10, false>), dim3(nseg), dim3(1024), 0, s, segs, list, nl, ns, nc, grad, res,
                       lr, out_idx, out_val);
  return hipGetLastError();
}

hipError_t launch_large(const LargePlan& pl, const Scratch& sc, const SegDesc* segs, const float* grad,
                        float* res, float lr, int32_t* out_idx, float* out_val, hipStream_t s, Prof* prof) {
  if (pl.n_large <= 0) return hipSuccess;
  // the layers' histograms and, behind them, the counters: one clearing launch per call
  uint32_t* counters = sc.ghist + (int64_t)pl.n_large * kHistStride;
  hipError_t e = launch_zero_u32(sc.ghist, (int64_t)pl.n_large * kHistStride + 16, s, prof);
  if (e != hipSuccess) return e;
  if (pl.n_sampled > 0) {
    ProfScope ps(prof, K_SAMPLE, s);
    if (pl.big_sample)
      hipLaunchKernelGGL((k_sample<true>), dim3(pl.n_sampled), dim3(1024), 0, s, segs, pl.sampled, pl.lsegs, grad,
                         res, lr, sc.lstate);
    else
      hipLaunchKernelGGL((k_sample<false>), dim3(pl.n_sampled), dim3(1024), 0, s, segs, pl.sampled, pl.lsegs, grad,
                         res, lr, sc.lstate);
  }
  {
    const int nl = (pl.n_tiles + kStreamLaunchTiles - 1) / kStreamLaunchTiles;
    ProfScope ps(prof, K_STREAM, s, nl);
    for (int t0 = 0; t0 < pl.n_tiles; t0 += kStreamLaunchTiles) {
      const int nt = pl.n_tiles - t0 < kStreamLaunchTiles ? pl.n_tiles - t0 : kStreamLaunchTiles;
      hipLaunchKernelGGL((k_stream<kStreamWaves, kStreamV>), dim3(nt), dim3(kStreamWaves * 64), kStreamLdsPad, s,
                         pl.tiles + t0, grad, res, lr, sc.lstate, sc.chunk_cnt, sc.slots, pl.slot, sc.ghist);
    }
  }
  {
    ProfScope ps(prof, K_CSCAN, s);
    hipLaunchKernelGGL(k_cscan, dim3(pl.n_large), dim3(1024), 0, s, segs, pl.lsegs, sc.lstate, sc.chunk_cnt,
                       pl.slot, sc.chunk_off, counters, sc.items);
  }
  if (pl.n_chunks > 0) {
    ProfScope ps(prof, K_CGATHER, s);
    hipLaunchKernelGGL(k_cgather, dim3((pl.n_chunks + 255) / 256), dim3(256), 0, s, pl.n_chunks, pl.chunk_lseg,
                       pl.lsegs, sc.lstate, sc.chunk_cnt, sc.chunk_off, sc.slots, pl.slot, sc.cand, segs, res);
  }
  const float* ng = nullptr;
  if (pl.n_cand_small[0] > 0) {
    ProfScope ps(prof, K_CSMALL0, s);
    hipLaunchKernelGGL((k_small<4, 1, true>), dim3(pl.n_cand_small[0]), dim3(256), 0, s, segs, pl.cand_small[0],
                       pl.lsegs, sc.lstate, sc.cand, ng, res, lr, out_idx, out_val);
  }
  if (pl.n_cand_small[1] > 0) {
    ProfScope ps(prof, K_CSMALL1, s);
    hipLaunchKernelGGL((k_small<4, 8, true>), dim3(pl.n_cand_small[1]), dim3(256), 0, s, segs, pl.cand_small[1],
                       pl.lsegs, sc.lstate, sc.cand, ng, res, lr, out_idx, out_val);
  }
  if (pl.n_cand_small[2] > 0) {
    ProfScope ps(prof, K_CSMALL2, s);
    hipLaunchKernelGGL((k_small<16, 10, true>), dim3(pl.n_cand_small[2]), dim3(1024), 0, s, segs,
                       pl.cand_small[2], pl.lsegs, sc.lstate, sc.cand, ng, res, lr, out_idx, out_val);
  }
  // candidate tiles first, then the workgroups of the fallback work list
  const int nct = pl.n_ctiles;
  const dim3 grid(nct + kDenseGrid), b(256);
  // the digit chosen from each level's histogram is computed by the workgroups of the next launch
  for (int level = 0; level < 3; ++level) {
    ProfScope ps(prof, K_HIST, s);
    if (level == 0)
      hipLaunchKernelGGL((k_hist<0>), grid, b, 0, s, nct, pl.ctiles, pl.tiles, sc.items, counters, pl.n_tiles,
                         pl.lsegs, segs, res, sc.cand, sc.lstate, sc.ghist);
    else if (level == 1)
      hipLaunchKernelGGL((k_hist<1>), grid, b, 0, s, nct, pl.ctiles, pl.tiles, sc.items, counters, pl.n_tiles,
                         pl.lsegs, segs, res, sc.cand, sc.lstate, sc.ghist);
    else
      hipLaunchKernelGGL((k_hist<2>), grid, b, 0, s, nct, pl.ctiles, pl.tiles, sc.items, counters, pl.n_tiles,
                         pl.lsegs, segs, res, sc.cand, sc.lstate, sc.ghist);
  }
  {
    ProfScope ps(prof, K_COUNT, s);
    hipLaunchKernelGGL(k_count, grid, b, 0, s, nct, pl.ctiles, pl.tiles, sc.items, counters, pl.n_tiles, res,
                       sc.cand, sc.lstate, sc.ghist, sc.tile_gt, sc.tile_eq);
  }
  {
    ProfScope ps(prof, K_SCAN, s);
    hipLaunchKernelGGL(k_scan, dim3(pl.n_large), dim3(1024), 0, s, pl.lsegs, sc.lstate, pl.n_tiles, sc.tile_gt,
                       sc.tile_eq);
  }
  {
    ProfScope ps(prof, K_EMIT, s);
    hipLaunchKernelGGL(k_emit, grid, b, 0, s, nct, pl.ctiles, pl.tiles, sc.items, counters, pl.n_tiles, pl.lsegs,
                       segs, res, sc.cand, sc.lstate, sc.tile_gt, sc.tile_eq, out_idx, out_val);
  }
  return hipGetLastError();
}

hipError_t launch_merge(int mode, const MergePlan& mp, int32_t* bounds, const SegDesc* segs, const int32_t* idx,
                        const float* val, int P, int64_t stride_k, float* out, const float* res,
                        int64_t res_stride, double* partials, double* out3, hipStream_t s, Prof* prof) {
  if (mp.n_mtiles <= 0) return hipSuccess;
  {
    ProfScope ps(prof, K_MERGE_BOUNDS, s);
    hipLaunchKernelGGL(k_merge_bounds, dim3(mp.n_bchunks, P), dim3(256), 0, s, mp.bchunks, segs, idx, stride_k,
                       mp.nb, bounds);
  }
  if (mode == MERGE_UPDATE) {
    ProfScope ps(prof, K_MERGE, s);
    hipLaunchKernelGGL((k_merge<false>), dim3(mp.n_mtiles), dim3(256), 0, s, mp.mtiles, segs, idx, val, P, stride_k,
                       mp.nb, bounds, out);
  } else if (mode == MERGE_APPLY) {
    ProfScope ps(prof, K_MERGE_APPLY, s);
    hipLaunchKernelGGL((k_merge<true>), dim3(mp.n_mtiles), dim3(256), 0, s, mp.mtiles, segs, idx, val, P, stride_k,
                       mp.nb, bounds, out);
  } else {
    {
      ProfScope ps(prof, K_DELTA_TILES, s);
      hipLaunchKernelGGL(k_delta_tiles, dim3(mp.n_mtiles), dim3(256), 0, s, mp.mtiles, segs, res, res_stride, idx,
                         val, P, stride_k, mp.nb, bounds, partials);
    }
    ProfScope ps(prof, K_DELTA_FINISH, s);
    hipLaunchKernelGGL(k_delta_finish, dim3(mp.n_layers), dim3(256), 0, s, segs, mp.seg_mtile0, partials, out3);
  }
  return hipGetLastError();
}

}  // namespace lags
