// HIP kernels (gfx950, wave64) of the per-layer error-compensated top-k sparsifier.
//
// What is computed (LAGS-SGD, Algorithm 1 lines 6-9, TopK of Eq. 4):
//   acc = residual + lr*grad; keep the k entries of largest |acc| (ties: lower index);
//   emit (index, acc) ascending; residual = acc with kept entries zeroed;
//   merge: update = (sum_p kept_p) / P.
//
// The order is that of key = bits(acc) & 0x7fffffff.  The k-th entry in the order (key
// descending, index ascending) fixes the kept set: key above its key T, or key == T and an index
// up to its index (equivalently: the first r entries equal to T in index order).
//
// Work layout: a wave owns a contiguous chunk of V*256 elements and walks it in V
// rounds; in a round lane i holds the 4 consecutive elements (round*256 + 4*i ..+3),
// so loads/stores are 16-byte vectors, coalesced over the wave, and index order is
// (round, lane, component).  Ordered compaction uses per-wave counts, a scan over waves
// (and over tiles for multi-block layers) and a wave prefix scan per round.
//
// Three routes, chosen per layer by size:
//   small  (d <= 8192): one workgroup, acc stays in registers between the single read of
//          grad/residual and the single write of the residual; exact select over linear bins
//          (k <= 256) or an exact radix select, digits of 11 + 10 + 10 key bits, LDS histograms.
//   large, sampled: a sample of 4096 or 16384 elements gives a threshold tau that, with high
//          probability, admits somewhat more than k entries.  One streaming pass writes acc
//          into the residual buffer and collects every entry with key >= tau (in index order)
//          into per-tile slots.  The finish counts them in buckets of the key range just above
//          tau.  If at least k were collected and no tile overflowed, the exact top k are among
//          them: the bucket counts name the bucket that holds the k-th largest key, its few
//          entries are ranked exactly, and one more pass over the slots emits the kept pairs.
//          The guess never changes the result: it is verified by the counts.
//   large, multi-pass: the radix select over the acc values in the residual buffer, multi-block
//          (layers too dense to sample; rejected guesses).
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

// Inclusive scan over the 64 lanes of a wave with data-parallel-primitive moves (no LDS
// traffic: measured 77 ns against 246 ns for the same scan with shuffles in a 16-wave
// workgroup): four shifts inside each row of 16 lanes, then the last lane of rows 0 and 2 is
// added to rows 1 and 3, then lane 31 to rows 2 and 3.  A lane without a source adds 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_add(uint32_t v) {
  return v + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x, int /*lane*/) {
  x = dpp_add<0x111, 0xF>(x);  // row_shr:1
  x = dpp_add<0x112, 0xF>(x);  // row_shr:2
  x = dpp_add<0x114, 0xF>(x);  // row_shr:4
  x = dpp_add<0x118, 0xF>(x);  // row_shr:8
  x = dpp_add<0x142, 0xA>(x);  // row_bcast:15 into rows 1 and 3
  x = dpp_add<0x143, 0xC>(x);  // row_bcast:31 into rows 2 and 3
  return x;
}

// Value of lane 63 in every lane (wave-uniform).
__device__ __forceinline__ uint32_t wave_last(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t x) { return wave_last(wave_incl_scan(x, 0)); }

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

enum { EMIT_FULL = 0, EMIT_ZERO = 1 };

// Ordered emission of a wave's chunk.  gt_before / eq_before: numbers of keys > T and
// == T that precede the chunk in the layer.  An element is kept if key > T, or key == T
// and fewer than `rtake` equal keys precede it; its output slot is the number of kept
// elements before it = gt_before + min(eq_before, rtake).
// EMIT_FULL: the chunk is residual data; it is written back completely (acc, kept entries
//            zeroed).  r = the chunk's residual.
// EMIT_ZERO: the residual already holds acc; only the kept entries are zeroed.  r = the
//            chunk's residual.
template <int V, int MODE>
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
    const uint32_t tot = wave_last(incl);
    const uint32_t excl = incl - packed;
    uint32_t gb = gt_before + (excl & 0xFFFFu);
    uint32_t eb = eq_before + (excl >> 16);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool sel = fg[c] || (fe[c] && eb < rtake);
      const uint32_t pos = gb + (eb < rtake ? eb : rtake);
      if (sel && pos < k) {  // pos < k always holds; the check keeps a wrong T from writing out of bounds
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

template <int NT>
__device__ __forceinline__ uint32_t block_max(uint32_t v, uint32_t* s_wt) {
  const int lane = lane_id(), w = threadIdx.x >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const uint32_t t = __shfl_xor(v, o, 64);
    v = t > v ? t : v;
  }
  __syncthreads();
  if (lane == 0) s_wt[w] = v;
  __syncthreads();
  uint32_t m = 0;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) m = s_wt[i] > m ? s_wt[i] : m;
  return m;
}

// Sum of a and of b over the workgroup (two barriers; s_tmp holds 2 * NT / 64 words).
template <int NT>
__device__ __forceinline__ void block_sum2(uint32_t& a, uint32_t& b, uint32_t* s_tmp) {
  constexpr int NW = NT / 64;
  const int lane = lane_id(), w = threadIdx.x >> 6;
  a = wave_sum(a);
  b = wave_sum(b);
  __syncthreads();
  if (lane == 0) { s_tmp[w] = a; s_tmp[NW + w] = b; }
  __syncthreads();
  uint32_t ta = 0, tb = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) { ta += s_tmp[i]; tb += s_tmp[NW + i]; }
  a = ta;
  b = tb;
}

// For a histogram of NT bins ordered by key, one bin count h per thread: the bins that hold
// the entries of ranks r1 and r2 (1-based, counted from the top bin downwards).
// s_out[0] = bin of r1, s_out[1] = rank of that entry inside the bin (0: the histogram holds
// fewer than r1 entries), s_out[2] = the bin's count; s_out[3], s_out[4] = bin and rank for r2.
// Three barriers; every thread may read s_out afterwards.
template <int NT>
__device__ __forceinline__ void find_two_ranks(uint32_t h, uint32_t r1, uint32_t r2, uint32_t* s_wt,
                                               uint32_t* s_out) {
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const uint32_t x = wave_incl_scan(h, lane);
  __syncthreads();
  if (lane == 63) s_wt[w] = x;
  if (tid < 5) s_out[tid] = 0u;
  __syncthreads();
  uint32_t off = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    const uint32_t t = s_wt[i];
    if (i < w) off += t;
    tot += t;
  }
  const uint32_t above = tot - (x + off);  // entries in the bins above this thread's
  if (above < r1 && r1 <= above + h) { s_out[0] = (uint32_t)tid; s_out[1] = r1 - above; s_out[2] = h; }
  if (above < r2 && r2 <= above + h) { s_out[3] = (uint32_t)tid; s_out[4] = r2 - above; }
  __syncthreads();
}

// Exact selection over keys held in registers by a whole workgroup when k <= NT: the k-th
// largest key T and the number of entries equal to T that belong to the top k.  Histograms over
// NT linear bins, which spread the top of the layer evenly (bins of exponent bits put it into a
// handful of LDS words whose atomics then serialise): first the per-thread maxima over the 2^26
// key steps below the largest key M give a floor F that at least k thread maxima reach; then
// the entries at or above F are binned over [F, M] and the bin that holds rank k is refined,
// log2(NT) key bits at a time, until it is one key wide.  Returns false (uniform over the
// workgroup, nothing decided) if k > NT or fewer than k thread maxima lie within 2^26 key steps
// of M: the caller then takes the radix select.  s_hist: NT words, s_wt: NT/64, s_out: 5.
template <int NT, int V>
__device__ __forceinline__ bool block_select_linear(const uint32_t (&a)[V][4], int n_w, int lane, uint32_t k,
                                                    uint32_t* s_hist, uint32_t* s_wt, uint32_t* s_out, uint32_t& T,
                                                    uint32_t& rtake) {
  constexpr int LOG = NT == 1024 ? 10 : 8;
  static_assert(NT == 1024 || NT == 256, "one bin per thread");
  if (k > (uint32_t)NT) return false;
  const int tid = threadIdx.x;
  uint32_t mx = 0u;
  bool any = false;
#pragma unroll
  for (int j = 0; j < V; ++j) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (j * 256 + lane * 4 + c < n_w) {
        const uint32_t key = a[j][c] & 0x7FFFFFFFu;
        mx = key > mx ? key : mx;
        any = true;
      }
    }
  }
  const uint32_t M = block_max<NT>(mx, s_wt);
  const uint32_t L1 = M > 0x03FFFFFFu ? M - 0x03FFFFFFu : 0u;
  s_hist[tid] = 0u;
  __syncthreads();
  if (any && mx >= L1) atomicAdd(&s_hist[(mx - L1) >> (26 - LOG)], 1u);
  __syncthreads();
  find_two_ranks<NT>(s_hist[tid], k, k, s_wt, s_out);
  if (s_out[1] == 0u) return false;
  uint32_t lo = L1 + (s_out[0] << (26 - LOG)), width = M - lo + 1u, want = k;
  int sh = 0;
  while (((width - 1u) >> sh) >= (uint32_t)NT) ++sh;
  for (;;) {  // uniform over the workgroup; the bin width shrinks by LOG bits per round
    __syncthreads();
    s_hist[tid] = 0u;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < V; ++j) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t key = a[j][c] & 0x7FFFFFFFu;
        if (j * 256 + lane * 4 + c < n_w && key >= lo && key - lo < width) atomicAdd(&s_hist[(key - lo) >> sh], 1u);
      }
    }
    __syncthreads();
    find_two_ranks<NT>(s_hist[tid], want, want, s_wt, s_out);
    if (s_out[1] == 0u) return false;  // cannot happen: the range held `want` entries
    lo += s_out[0] << sh;
    want = s_out[1];
    if (sh == 0) break;
    width = 1u << sh;
    sh = sh > LOG ? sh - LOG : 0;
  }
  T = lo;
  rtake = want;
  return true;
}

// ------------------------------------------------------------------ small ----
// One workgroup per layer; the values live in registers between the single read and the write.
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
  __shared__ uint32_t s_out[5];
  __shared__ uint32_t s_wg[NW], s_we[NW];

  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const SegDesc sd = segs[list[blockIdx.x]];
  const int n_w = sd.d - w * CH;
  float* r = res + sd.offset + (int64_t)w * CH;
  const float* g = grad + sd.offset + (int64_t)w * CH;
  const bool vec = aligned16(g, r);

  uint32_t a[V][4];
  load_acc<V>(g, r, n_w, lr, vec, lane, a);

  uint32_t T, rtake;
  if (!block_select_linear<NT, V>(a, n_w, lane, (uint32_t)sd.k, s_hist, s_wt, s_out, T, rtake))  // uniform
    block_radix_select<NT, V>(a, n_w, lane, (uint32_t)sd.k, s_hist, s_wt, s_sel, T, rtake);

  uint32_t cg, ce;
  lane_count<V>(a, n_w, lane, T, cg, ce);
  cg = wave_sum(cg);
  ce = wave_sum(ce);
  __syncthreads();
  if (lane == 0) { s_wg[w] = cg; s_we[w] = ce; }
  __syncthreads();
  uint32_t gb = 0, eb = 0;
  for (int i = 0; i < w; ++i) { gb += s_wg[i]; eb += s_we[i]; }
  wave_emit<V, EMIT_FULL>(a, n_w, lane, T, rtake, gb, eb, (uint32_t)sd.k, w * CH, out_idx + sd.out_offset,
                          out_val + sd.out_offset, r, vec);
}

// ------------------------------------------------------------------ prep -----
// Finds, in a histogram whose bins are ordered by key, the bin that holds the entry of rank
// `rank` (1-based, counted from the top bin downwards) and that entry's rank inside the bin.
// Returns false if the histogram holds fewer than `rank` entries.  Contains barriers; every
// thread gets the result.
template <int NT>
__device__ __forceinline__ bool find_rank(const uint32_t* hist, int nb, uint32_t rank, uint32_t* s_wt,
                                          uint32_t* s_sel, uint32_t& bin, uint32_t& rank_in_bin) {
  __syncthreads();
  if (threadIdx.x == 0) { s_sel[0] = 0u; s_sel[1] = 0u; }
  __syncthreads();
  block_find_bucket<NT>(hist, nb, rank, s_wt, s_sel);
  bin = s_sel[0];
  rank_in_bin = s_sel[1];
  return rank_in_bin != 0u;
}

// Workgroup of the threshold guess: 4 waves; a thread holds V * 4 sample keys, V = 16 for the
// full sample of kSamplePieces pieces and V = 4 for the short sample of kSamplePiecesSmall.
// Small workgroups, so that many layers are guessed at once: a CU holds four of them side by
// side, and what bounds the kernel is then the scattered reads of the samples themselves.
constexpr int kPrepThreads = 256;
constexpr int kPrepV = kSampleMax / (kPrepThreads * 4);
constexpr int kPrepVSmall = kSamplePiecesSmall * kSamplePiece / (kPrepThreads * 4);
static_assert(kPrepV * kPrepThreads * 4 == kSampleMax, "every sample slot has a thread");
static_assert(kPrepVSmall * kPrepThreads * 4 == kSamplePiecesSmall * kSamplePiece && kPrepVSmall % 2 == 0,
              "every slot of the short sample has a thread");

// Keys of the sample: 16 V pieces of kSamplePiece consecutive elements; a wave round of 64
// lanes x 4 elements covers 4 pieces, wave w owns the pieces [4 V w, 4 V w + 4 V).
// The loads of half the rounds are issued before any of them is used, from addresses that are
// valid whether or not the sample slot exists (a slot that does not, or that would cross the
// layer's end, reads the layer's first elements and is then set to key 0): no branch separates
// the loads, so their latencies overlap; two halves, so that the registers of the loads in
// flight and of the keys leave room for four waves per SIMD.  Large layers hold more than 4
// elements.
template <int V>
__device__ __forceinline__ void sample_keys(const LargeSeg& ls, int li, const SegDesc& sd,
                                            const float* __restrict__ g, const float* __restrict__ r, bool vec,
                                            float lr, int lane, int w, uint32_t (&a)[V][4]) {
  constexpr int H = V / 2;
  constexpr int LP = kSamplePiece / 4;         // lanes per piece
  constexpr int PR = 64 / LP;                  // pieces per wave round
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    int e[H];
    bool have[H];
#pragma unroll
    for (int jj = 0; jj < H; ++jj) {
      const int j = half * H + jj;
      const int piece = w * (V * PR) + j * PR + (lane / LP);
      int start = piece * ls.sample_stride;
      if (ls.sample_stride > kSamplePiece)
        start += (int)(mix32((uint32_t)piece * 0x9E3779B9u + (uint32_t)li) %
                       (uint32_t)(ls.sample_stride - kSamplePiece + 1));
      start &= ~3;
      e[jj] = start + (lane % LP) * 4;
      have[jj] = piece < ls.sample_pieces && e[jj] >= 0 && e[jj] + 3 < sd.d;
      if (!have[jj]) e[jj] = 0;
    }
    if (vec) {
      float4 gv[H], rv[H];
#pragma unroll
      for (int jj = 0; jj < H; ++jj) {
        gv[jj] = *reinterpret_cast<const float4*>(g + e[jj]);
        rv[jj] = *reinterpret_cast<const float4*>(r + e[jj]);
      }
#pragma unroll
      for (int jj = 0; jj < H; ++jj) {
        const int j = half * H + jj;
        a[j][0] = acc_bits(gv[jj].x, rv[jj].x, lr);
        a[j][1] = acc_bits(gv[jj].y, rv[jj].y, lr);
        a[j][2] = acc_bits(gv[jj].z, rv[jj].z, lr);
        a[j][3] = acc_bits(gv[jj].w, rv[jj].w, lr);
      }
    } else {
#pragma unroll
      for (int jj = 0; jj < H; ++jj) {
        const int j = half * H + jj;
        float gs[4], rs[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          gs[c] = g[e[jj] + c];
          rs[c] = r[e[jj] + c];
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) a[j][c] = acc_bits(gs[c], rs[c], lr);
      }
    }
#pragma unroll
    for (int jj = 0; jj < H; ++jj) {
      const int j = half * H + jj;
#pragma unroll
      for (int c = 0; c < 4; ++c) a[j][c] = have[jj] ? (a[j][c] & 0x7FFFFFFFu) : 0u;
    }
  }
}

// Threshold guess for one large layer: form acc on up to 16 V pieces of 64 consecutive elements
// spread over the layer (with a hashed offset inside each stride); tau is a key that at least
// `sample_rank` sample keys reach (and few more), t_est one that at least `sample_rank_hi`
// reach: the sample's estimate of the layer's k-th largest key.  Any value would be correct
// (the guess is verified by counting); a good one keeps the candidates few.  Missing sample
// slots count as key 0.
//
// The two keys come from two histograms over NT linear bins, which spread the top of the
// sample evenly (bins of exponent bits would put it all into a handful of LDS words):
// first the per-thread maxima over the 2^26 key steps below the largest sample key M, which
// gives a floor F that at least `sample_rank` thread maxima reach; then the sample entries at
// or above F over [F, M].  The lower edge of the bin that holds a rank is returned; where that
// bin holds clearly more entries than the rank needs, the rank is resolved inside it.  Ranks
// above NT (dense layers) and samples whose top spans more than 2^26 key steps take an exact
// radix select instead.
template <int V>
__device__ __forceinline__ void sample_layer(const LargeSeg& ls, int li, const SegDesc& sd,
                                             const float* __restrict__ grad, const float* __restrict__ res,
                                             float lr, uint32_t* s_hist, uint32_t* s_wt, uint32_t* s_sel,
                                             uint32_t* s_out, uint32_t& tau, uint32_t& t_est) {
  constexpr int NT = kPrepThreads;
  constexpr int LOG = 8;                      // log2(NT): key bits resolved per histogram
  static_assert((1 << LOG) == NT, "one bin per thread");
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const float* g = grad + sd.offset;
  const float* r = res + sd.offset;
  const bool vec = aligned16(g, r);
  const uint32_t rank = (uint32_t)ls.sample_rank, rank_hi = (uint32_t)ls.sample_rank_hi;
  uint32_t a[V][4];
  sample_keys<V>(ls, li, sd, g, r, vec, lr, lane, w, a);
  uint32_t mx = 0u;
#pragma unroll
  for (int j = 0; j < V; ++j) {
#pragma unroll
    for (int c = 0; c < 4; ++c) mx = a[j][c] > mx ? a[j][c] : mx;
  }
  const uint32_t M = block_max<NT>(mx, s_wt);
  bool fast = rank <= (uint32_t)NT;  // uniform over the workgroup
  uint32_t F = 0u;
  if (fast) {
    const uint32_t L1 = M > 0x03FFFFFFu ? M - 0x03FFFFFFu : 0u;
    s_hist[tid] = 0u;
    __syncthreads();
    if (mx >= L1) atomicAdd(&s_hist[(mx - L1) >> (26 - LOG)], 1u);
    __syncthreads();
    find_two_ranks<NT>(s_hist[tid], rank, rank, s_wt, s_out);
    fast = s_out[1] != 0u;
    F = L1 + (s_out[0] << (26 - LOG));
  }
  if (fast) {
    int s2 = 0;
    while (((M - F) >> s2) >= (uint32_t)NT) ++s2;
    __syncthreads();
    s_hist[tid] = 0u;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < V; ++j) {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (a[j][c] >= F) atomicAdd(&s_hist[(a[j][c] - F) >> s2], 1u);
    }
    __syncthreads();
    // at least `rank` entries reach F, so both ranks are found
    find_two_ranks<NT>(s_hist[tid], rank, rank_hi, s_wt, s_out);
    tau = F + (s_out[0] << s2);
    t_est = F + (s_out[3] << s2);
    // If the bin of tau holds clearly more sample entries than the rank needs (keys that lie
    // closer together than the bins are wide: quantised or narrow data), its lower edge would
    // admit them all: resolve the rank inside the bin, NT finer bins at a time.
    uint32_t rib = s_out[1];
    uint32_t extra = rib != 0u ? s_out[2] - rib : 0u;
    while (s2 > 0 && extra > 4u) {  // uniform over the workgroup
      const uint32_t lo = tau, width = 1u << s2;
      s2 = s2 > LOG ? s2 - LOG : 0;
      __syncthreads();
      s_hist[tid] = 0u;
      __syncthreads();
#pragma unroll
      for (int j = 0; j < V; ++j) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (a[j][c] >= lo && a[j][c] - lo < width) atomicAdd(&s_hist[(a[j][c] - lo) >> s2], 1u);
      }
      __syncthreads();
      find_two_ranks<NT>(s_hist[tid], rib, rib, s_wt, s_out);
      if (s_out[1] == 0u) break;  // cannot happen: the bin held `rib` entries
      tau = lo + (s_out[0] << s2);
      rib = s_out[1];
      extra = s_out[2] - rib;
    }
  } else {
    uint32_t rtake;
    block_radix_select<NT, V>(a, V * 256, lane, rank, s_hist, s_wt, s_sel, tau, rtake);
    block_radix_select<NT, V>(a, V * 256, lane, rank_hi, s_hist, s_wt, s_sel, t_est, rtake);
  }
  if (t_est < tau) t_est = tau;
}

// One workgroup per large layer: resets the layer's per-call state (and, when the multi-pass
// kernels will run, their histograms and work counter) and guesses the threshold of a sampled
// layer.
__global__ __launch_bounds__(kPrepThreads) __attribute__((amdgpu_waves_per_eu(4, 8))) void k_prep(const SegDesc* __restrict__ segs,
                                                       const LargeSeg* __restrict__ lsegs,
                                                       const float* __restrict__ grad,
                                                       const float* __restrict__ res, float lr,
                                                       LState* __restrict__ lstate, uint32_t* __restrict__ ghist,
                                                       uint32_t* __restrict__ counters, int chain) {
  __shared__ uint32_t s_hist[kBins0];
  __shared__ uint32_t s_wt[16];
  __shared__ uint32_t s_sel[2];
  __shared__ uint32_t s_out[5];
  const int li = blockIdx.x, tid = threadIdx.x;
  const LargeSeg ls = lsegs[li];
  if (chain) {
    static_assert(kHistStride % (4 * kPrepThreads) == 0, "16-byte stores clear a layer's histograms");
    for (int i = tid; i < kHistStride / 4; i += kPrepThreads)
      reinterpret_cast<uint4*>(ghist + (int64_t)li * kHistStride)[i] = make_uint4(0u, 0u, 0u, 0u);
    if (li == 0 && tid < 16) counters[tid] = 0u;
  }
  if (!ls.sampled) {  // uniform over the workgroup
    if (tid == 0) {
      LState st = {};
      st.mode = MODE_DENSE;
      st.route = 3u;
      lstate[li] = st;
    }
    return;
  }
  const SegDesc sd = segs[ls.seg];
  uint32_t tau, t_est;
  if (ls.sample_pieces <= kSamplePiecesSmall)  // uniform over the workgroup
    sample_layer<kPrepVSmall>(ls, li, sd, grad, res, lr, s_hist, s_wt, s_sel, s_out, tau, t_est);
  else
    sample_layer<kPrepV>(ls, li, sd, grad, res, lr, s_hist, s_wt, s_sel, s_out, tau, t_est);
  if (tid == 0) {
    // bucket width: the distance from tau to the estimate of the k-th largest key spans 512 to
    // 1023 buckets, so the 4096 buckets reach four to eight times that distance above tau
    const uint32_t delta = t_est - tau;
    uint32_t shift = 0;
    while ((delta >> shift) >= 1024u) ++shift;
    const uint64_t top = (uint64_t)tau + ((uint64_t)kFineBins << shift);
    LState st = {};
    st.tau = tau;
    st.t_zero = t_est;
    st.tau_top = top > 0x80000000ull ? 0x80000000u : (uint32_t)top;  // keys are below 2^31
    st.shift = shift;
    st.mode = MODE_DENSE;
    lstate[li] = st;
  }
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
// and marks the tile as overflowed), and collected entries with key >= t_zero are replaced by
// zero in `a`.  FULL: the wave's chunk is complete, no bounds checks.
template <int NW, int V, bool FULL>
__device__ __forceinline__ void stream_collect(uint32_t (&a)[V][4], int n_w, int lane, int w, uint32_t tau,
                                               uint32_t t_zero, int32_t idx0, uint2* __restrict__ slot, int nslot,
                                               uint32_t* __restrict__ cnt, uint32_t* s_cnt) {
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
      // slot of the lane's first candidate of this round, then one predicated store per component
      uint32_t pos = base + mbcnt64(m[j][0]) + mbcnt64(m[j][1]) + mbcnt64(m[j][2]) + mbcnt64(m[j][3]);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t key = a[j][c] & 0x7FFFFFFFu;
        const bool f = FULL ? key >= tau : ((key >= tau) & (e + c < n_w));
        const bool put = f & (pos < (uint32_t)nslot);
        if (put) slot[pos] = make_uint2((uint32_t)(idx0 + e + c), a[j][c]);
        // an entry at or above t_zero is expected to be kept: its residual is written as zero
        // right here, with the rest of its line (its value is safe in the slot); the finish
        // corrects the entries for which that expectation turns out wrong.  A scattered 4-byte
        // write later costs about as much as a whole line of this pass.
        a[j][c] = (put & (key >= t_zero)) ? 0u : a[j][c];
        pos += f ? 1u : 0u;
      }
      base += tot;
    }
  }
}

// The one pass over grad and residual of every large layer: acc = residual + lr*grad is
// written into the residual buffer (it is the final residual everywhere but at the k kept
// entries).  Tiles of sampled layers also collect, in index order, the entries with
// key >= tau into the tile's slots; tiles of the other layers add to the layer's histogram of
// key bits 30..20.  Both arrays are touched exactly once, so full aligned tiles use
// non-temporal 16-byte loads and stores.  The launch adds kStreamLdsPad bytes of unused
// dynamic LDS per workgroup to cap the workgroups per CU.  The pass issues no global atomics
// for sampled layers (same-address atomics cost 0.06-0.2 us each on this chip: one per tile
// on a per-layer counter measured 7x the whole pass).
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
  uint32_t tau = 0, t_zero = 0;
  if (collect) {
    tau = lstate[td.seg].tau;
    t_zero = lstate[td.seg].t_zero;
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
    if (fast) stream_collect<NW, V, true>(a, n_w, lane, w, tau, t_zero, idx0, slot, nslot, cnt, s_cnt);
    else stream_collect<NW, V, false>(a, n_w, lane, w, tau, t_zero, idx0, slot, nslot, cnt, s_cnt);
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

// ------------------------------------------------------------------ finish ---
// After the streaming pass a sampled layer's candidates sit in its tiles' slots (index order
// inside a tile, tiles in index order).  The finish
//   counts    the candidates in kFineBins buckets of 2^shift key steps above tau (those at or
//             above tau_top, the end of the buckets, in one number);
//   decides   whether the guess held (at least k candidates, no tile overflowed) and which
//             bucket b* holds the k-th largest key, so that every candidate above b* is kept
//             and k_rem of the entries in b* (the "band", at most kBandCap) are;
//   phase A   counts per wave chunk (8 tiles) the candidates above b* and collects the band;
//   selects   among the band the entry of rank k_rem in the order (key descending, index
//             ascending): its key T and index I fix the kept set, key > T or key == T and index <= I;
//   phase B   writes the kept pairs in index order (position = kept entries of the earlier wave
//             chunks + kept band entries with a smaller index + rank inside the wave chunk) and
//             zeroes their residual.
// Layers of up to kFusedTiles tiles (kFusedTilesShared in tables that hold larger layers
// anyway) do all of it in one workgroup (k_finish; 256 threads up to kFinishSmallTiles tiles,
// 1024 above).  Larger ones take
// one launch per step: k_group_h (partial bucket counts per 256 tiles), k_finish (decides),
// k_group_a over groups of 64 tiles, k_group_p (one workgroup per layer: selects, turns the
// counts into output positions), k_group_b over the groups again.  Work that every group would
// repeat is done once per layer: hundreds of workgroups reading the same few kilobytes at the
// same time queue up at the cache channels that hold them (measured 30 us instead of 10 for the
// 392 groups of a 100 M-element layer).  No workgroup ever waits for another one, and nothing is added
// with global atomics.

// A wave's view of the slots of up to kWaveTiles consecutive tiles as one flat, index-ordered
// list.  The tiles' exclusive counts are wave-uniform (scalar registers).
struct WaveChunk {
  int c0;                      // first tile (chunk number)
  uint32_t pre[kWaveTiles];    // entries of the tiles before tile c0 + j
  uint32_t total;              // entries of all its tiles
};

__device__ __forceinline__ WaveChunk wc_open(int c0, int c_end, const uint32_t* __restrict__ chunk_cnt, int nslot,
                                             int lane) {
  uint32_t cnt = 0;
  if (lane < kWaveTiles && c0 + lane < c_end) {
    cnt = chunk_cnt[c0 + lane];
    cnt = cnt < (uint32_t)nslot ? cnt : (uint32_t)nslot;  // an overflowed tile rejects the layer; stay in bounds anyway
  }
  WaveChunk wc;
  wc.c0 = c0;
  uint32_t run = 0;
#pragma unroll
  for (int j = 0; j < kWaveTiles; ++j) {
    wc.pre[j] = run;
    run += (uint32_t)__builtin_amdgcn_readlane((int)cnt, j);
  }
  wc.total = run;
  return wc;
}

// Entry e < total of the flat list (e may differ per lane): its tile is the last one whose
// exclusive count is <= e (the counts are non-decreasing, so that is the number of such tiles
// after the first).
__device__ __forceinline__ uint2 wc_entry(const WaveChunk& wc, uint32_t e, const uint2* __restrict__ slots,
                                          int nslot) {
  uint32_t tile = 0, p0 = 0;
#pragma unroll
  for (int j = 1; j < kWaveTiles; ++j) {
    const bool ge = e >= wc.pre[j];
    tile += ge ? 1u : 0u;
    p0 = ge ? wc.pre[j] : p0;
  }
  return slots[(int64_t)(wc.c0 + (int)tile) * nslot + (e - p0)];
}

// Calls f(entry, live) for the wave chunk's entries, 64 at a time in index order, all lanes
// taking part (live = the lane holds an entry).  Two loads are issued before the first is used.
template <typename F>
__device__ __forceinline__ void wc_for_each(const WaveChunk& wc, const uint2* __restrict__ slots, int nslot,
                                            int lane, F f) {
  for (uint32_t base = 0; base < wc.total; base += 128) {  // wave-uniform trip count
    const bool two = base + 64 < wc.total;                 // wave-uniform
    const bool live0 = base + lane < wc.total, live1 = base + 64 + lane < wc.total;
    const uint2 e0 = wc_entry(wc, live0 ? base + lane : wc.total - 1, slots, nslot);
    uint2 e1 = make_uint2(0u, 0u);
    if (two) e1 = wc_entry(wc, live1 ? base + 64 + lane : wc.total - 1, slots, nslot);
    f(e0, live0);
    if (two) f(e1, live1);
  }
}

// Up to kWaveChunks wave chunks of one wave, walked together.  The first 128 entries of every
// chunk are loaded once, all loads in flight together, and stay in registers for the three
// passes (a chunk of a layer that keeps 0.1 % holds one to two hundred entries); what a chunk
// holds beyond that is read again in every pass.  Chunks without entries cost nothing.
constexpr int kWaveChunks = 4;
struct WaveEntries {
  uint2 e0[kWaveChunks], e1[kWaveChunks];  // entries lane and 64 + lane of each chunk
};

__device__ __forceinline__ void wc_load4(const WaveChunk (&wc)[kWaveChunks], const uint2* __restrict__ slots,
                                         int nslot, int lane, WaveEntries& we) {
#pragma unroll
  for (int i = 0; i < kWaveChunks; ++i) {
    const uint32_t n = wc[i].total;  // wave-uniform
    we.e0[i] = make_uint2(0u, 0u);
    we.e1[i] = make_uint2(0u, 0u);
    if (n > 0u) we.e0[i] = wc_entry(wc[i], (uint32_t)lane < n ? (uint32_t)lane : n - 1u, slots, nslot);
    if (n > 64u) we.e1[i] = wc_entry(wc[i], 64u + lane < n ? 64u + lane : n - 1u, slots, nslot);
  }
}

// Calls f(i, entry, live) chunk by chunk in index order, all lanes taking part.
template <typename F>
__device__ __forceinline__ void wc_for_each4(const WaveChunk (&wc)[kWaveChunks], const WaveEntries& we,
                                             const uint2* __restrict__ slots, int nslot, int lane, F f) {
#pragma unroll
  for (int i = 0; i < kWaveChunks; ++i) {
    const uint32_t n = wc[i].total;
    if (n > 0u) f(i, we.e0[i], (uint32_t)lane < n);
    if (n > 64u) f(i, we.e1[i], 64u + lane < n);
    for (uint32_t base = 128; base < n; base += 128) {  // wave-uniform trip count
      const bool two = base + 64 < n;
      const bool live0 = base + lane < n, live1 = base + 64 + lane < n;
      const uint2 x0 = wc_entry(wc[i], live0 ? base + lane : n - 1u, slots, nslot);
      uint2 x1 = make_uint2(0u, 0u);
      if (two) x1 = wc_entry(wc[i], live1 ? base + 64 + lane : n - 1u, slots, nslot);
      f(i, x0, live0);
      if (two) f(i, x1, live1);
    }
  }
}

// What the three passes over the candidates do with one entry (all lanes of the wave call them
// together; live = the lane holds an entry).
// Counting pass: the entry's bucket in the LDS histogram s_fine; n_top counts the candidates
// at or above tau_top (wave-uniform).
__device__ __forceinline__ void entry_count(uint2 en, bool live, uint32_t tau, uint32_t tau_top, uint32_t shift,
                                            uint32_t* s_fine, uint32_t& n_top) {
  const uint32_t key = en.y & 0x7FFFFFFFu;
  const bool top = key >= tau_top;
  n_top += (uint32_t)__popcll(__ballot(live && top));
  if (live && !top) {
    // slots hold keys in [tau, tau_top) here; the clamps only keep a corrupted entry inside the array
    const uint32_t b = key >= tau ? (key - tau) >> shift : 0u;
    atomicAdd(&s_fine[b < (uint32_t)kFineBins ? b : (uint32_t)kFineBins - 1u], 1u);
  }
}

// Phase A: n_gt counts the candidates above bucket b* (wave-uniform); the entries of bucket b*
// are appended to band[0 .. cap) through the LDS counter *s_nband.
__device__ __forceinline__ void entry_phase_a(uint2 en, bool live, uint32_t tau, uint32_t tau_top, uint32_t shift,
                                              uint32_t bstar, uint2* band, uint32_t cap, uint32_t* s_nband,
                                              uint32_t& n_gt) {
  const uint32_t key = en.y & 0x7FFFFFFFu;
  const bool top = key >= tau_top;
  const uint32_t b = (key - tau) >> shift;
  n_gt += (uint32_t)__popcll(__ballot(live && (top || b > bstar)));
  if (live && !top && b == bstar) {
    const uint32_t pos = atomicAdd(s_nband, 1u);
    if (pos < cap) band[pos] = en;
  }
}

// Phase B: the kept entries go to out[pos0 ...] in index order (pos0 advances).  The streaming
// pass wrote zero for the entries with key >= t_zero and acc for the others, so the residual is
// written only where that differs from the outcome: zero for kept entries below t_zero, acc
// for dropped entries at or above it.  Positions are checked against k so that no state can
// write out of bounds.
__device__ __forceinline__ void entry_phase_b(uint2 en, bool live, uint32_t T, uint32_t I, uint32_t t_zero,
                                              uint32_t& pos0, uint32_t k, int32_t d, int32_t* __restrict__ oi,
                                              float* __restrict__ ov, float* __restrict__ rl) {
  const uint32_t key = en.y & 0x7FFFFFFFu;
  const bool keep = live && (key > T || (key == T && en.x <= I));
  const bool zeroed = key >= t_zero;  // what the streaming pass assumed
  const uint64_t mk = __ballot(keep);
  const uint32_t pos = pos0 + mbcnt64(mk);
  if (live && en.x < (uint32_t)d) {
    if (keep && pos < k) {
      oi[pos] = (int32_t)en.x;
      ov[pos] = __uint_as_float(en.y);
    }
    if (keep && !zeroed) rl[en.x] = 0.0f;
    if (!keep && zeroed) rl[en.x] = __uint_as_float(en.y);
  }
  pos0 += (uint32_t)__popcll(mk);
}

// The passes over one wave chunk.
__device__ __forceinline__ uint32_t wc_count(const WaveChunk& wc, const uint2* __restrict__ slots, int nslot,
                                             uint32_t tau, uint32_t tau_top, uint32_t shift, uint32_t* s_fine,
                                             int lane) {
  uint32_t n_top = 0;
  wc_for_each(wc, slots, nslot, lane,
              [&](uint2 en, bool live) { entry_count(en, live, tau, tau_top, shift, s_fine, n_top); });
  return n_top;
}

__device__ __forceinline__ uint32_t wc_phase_a(const WaveChunk& wc, const uint2* __restrict__ slots, int nslot,
                                               uint32_t tau, uint32_t tau_top, uint32_t shift, uint32_t bstar,
                                               uint2* band, uint32_t cap, uint32_t* s_nband, int lane) {
  uint32_t n_gt = 0;
  wc_for_each(wc, slots, nslot, lane, [&](uint2 en, bool live) {
    entry_phase_a(en, live, tau, tau_top, shift, bstar, band, cap, s_nband, n_gt);
  });
  return n_gt;
}

// The band entry of rank k_rem (1-based) in the order (key descending, index ascending):
// s_ti[0] = its key T, s_ti[1] = its index I.  The band has m <= kBandCap entries in LDS, all
// with keys in [lo, lo + 2^shift); 1 <= k_rem <= m.  A histogram over 1024 sub-buckets names
// the sub-bucket of that entry; the sub-bucket's entries (usually a handful) are copied out and
// each counts how many of them precede it.  s_bins: kFineBins words (1024 sub-bucket counts,
// then up to kFineBins / 2 copies).  Ends with a barrier.
template <int NT>
__device__ __forceinline__ void band_select(const uint2* s_band, uint32_t m, uint32_t k_rem, uint32_t lo,
                                            uint32_t shift, uint32_t* s_bins, uint32_t* s_wt, uint32_t* s_sel,
                                            uint32_t* s_ti) {
  const uint32_t s1 = shift > 10u ? shift - 10u : 0u;
  __syncthreads();
  for (int i = threadIdx.x; i < 1024; i += NT) s_bins[i] = 0u;
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < m; i += NT) {
    const uint32_t sub = ((s_band[i].y & 0x7FFFFFFFu) - lo) >> s1;
    atomicAdd(&s_bins[sub < 1023u ? sub : 1023u], 1u);
  }
  uint32_t b1, r1;
  if (find_rank<NT>(s_bins, 1024, k_rem, s_wt, s_sel, b1, r1)) {  // uniform over the workgroup
    __syncthreads();
    if (threadIdx.x == 0) s_sel[0] = 0u;  // number of copies
    __syncthreads();
    uint2* s_copy = reinterpret_cast<uint2*>(s_bins);
    constexpr uint32_t kCopies = kFineBins / 2;  // s_bins holds kFineBins words
    for (uint32_t i = threadIdx.x; i < m; i += NT) {
      const uint2 en = s_band[i];
      const uint32_t sub = ((en.y & 0x7FFFFFFFu) - lo) >> s1;
      if ((sub < 1023u ? sub : 1023u) == b1) {
        const uint32_t at = atomicAdd(&s_sel[0], 1u);
        if (at < kCopies) s_copy[at] = en;
      }
    }
    __syncthreads();
    const uint32_t c = s_sel[0];
    if (c <= kCopies) {  // uniform over the workgroup
      for (uint32_t i = threadIdx.x; i < c; i += NT) {
        const uint2 en = s_copy[i];
        const uint32_t key = en.y & 0x7FFFFFFFu;
        uint32_t before = 0;
        for (uint32_t q = 0; q < c; ++q) {
          const uint2 o = s_copy[q];
          const uint32_t ok = o.y & 0x7FFFFFFFu;
          before += (ok > key) || (ok == key && o.x < en.x);
        }
        if (before + 1u == r1) { s_ti[0] = key; s_ti[1] = en.x; }
      }
    } else {  // thousands of entries in one sub-bucket (ties): count inside the band itself
      for (uint32_t i = threadIdx.x; i < m; i += NT) {
        const uint2 en = s_band[i];
        const uint32_t key = en.y & 0x7FFFFFFFu;
        const uint32_t sub = (key - lo) >> s1;
        if ((sub < 1023u ? sub : 1023u) != b1) continue;
        uint32_t before = 0;
        for (uint32_t q = 0; q < m; ++q) {
          const uint2 o = s_band[q];
          const uint32_t ok = o.y & 0x7FFFFFFFu;
          const uint32_t osub = (ok - lo) >> s1;
          before += ((osub < 1023u ? osub : 1023u) == b1) && ((ok > key) || (ok == key && o.x < en.x));
        }
        if (before + 1u == r1) { s_ti[0] = key; s_ti[1] = en.x; }
      }
    }
  }
  __syncthreads();
}

// Kept band entries whose index is below idx0 (wave-uniform result).
__device__ __forceinline__ uint32_t band_kept_before(const uint2* s_band, uint32_t m, uint32_t T, uint32_t I,
                                                     uint32_t idx0, int lane) {
  uint32_t c = 0;
  for (uint32_t i = lane; i < m; i += 64) {
    const uint2 en = s_band[i];
    const uint32_t key = en.y & 0x7FFFFFFFu;
    c += (en.x < idx0) && (key > T || (key == T && en.x <= I));
  }
  return wave_sum(c);
}

__device__ __forceinline__ void wc_phase_b(const WaveChunk& wc, const uint2* __restrict__ slots, int nslot,
                                           uint32_t T, uint32_t I, uint32_t t_zero, uint32_t pos0, uint32_t k,
                                           int32_t d, int32_t* __restrict__ oi, float* __restrict__ ov,
                                           float* __restrict__ rl, int lane) {
  wc_for_each(wc, slots, nslot, lane,
              [&](uint2 en, bool live) { entry_phase_b(en, live, T, I, t_zero, pos0, k, d, oi, ov, rl); });
}

// Gives the entries that the streaming pass zeroed (slotted, key >= t_zero) their acc back:
// a layer whose guess is rejected is selected from the acc values in the residual buffer.
template <int NT>
__device__ __forceinline__ void restore_layer(const LargeSeg& ls, const SegDesc& sd, uint32_t t_zero,
                                              const uint32_t* __restrict__ chunk_cnt,
                                              const uint2* __restrict__ slots, int nslot, float* __restrict__ res) {
  const int lane = lane_id(), w = threadIdx.x >> 6;
  const int nwc = (ls.chunk_end - ls.chunk_begin + kWaveTiles - 1) / kWaveTiles;
  float* rl = res + sd.offset;
  for (int q = w; q < nwc; q += NT / 64) {
    const WaveChunk wc = wc_open(ls.chunk_begin + q * kWaveTiles, ls.chunk_end, chunk_cnt, nslot, lane);
    wc_for_each(wc, slots, nslot, lane, [&](uint2 en, bool live) {
      if (live && (en.y & 0x7FFFFFFFu) >= t_zero && en.x < (uint32_t)sd.d) rl[en.x] = __uint_as_float(en.y);
    });
  }
  __syncthreads();  // the workgroup's own later reads of the residual see these writes
}

// Exact selection of one layer by one workgroup from the acc values in the residual buffer:
// three histogram passes over the layer (digits of 11 + 10 + 10 key bits), then one ordered
// emission pass.  Slow (one workgroup walks the whole layer four times); used only where a
// guess was rejected and the multi-pass kernels are not enqueued.
template <int NT>
__device__ __forceinline__ void rescue_layer(const SegDesc& sd, float* __restrict__ res,
                                             int32_t* __restrict__ out_idx, float* __restrict__ out_val,
                                             uint32_t* s_hist, uint32_t* s_wt, uint32_t* s_sel) {
  const int tid = threadIdx.x, lane = lane_id();
  float* rl = res + sd.offset;
  int32_t* oi = out_idx + sd.out_offset;
  float* ov = out_val + sd.out_offset;
  uint32_t prefix = 0, mask = 0, k_rem = (uint32_t)sd.k;
  for (int level = 0; level < 3; ++level) {
    const int shift = level == 0 ? 20 : (level == 1 ? 10 : 0);
    const int nb = level == 0 ? kBins0 : kBins12;
    __syncthreads();
    for (int i = tid; i < nb; i += NT) s_hist[i] = 0u;
    __syncthreads();
    for (int64_t base = 0; base < sd.d; base += NT) {  // uniform trip count: the peeled add needs whole waves
      const int64_t i = base + tid;  // 64 bits: base + NT may pass 2^31
      uint32_t b = 0xFFFFFFFFu;
      if (i < sd.d) {
        const uint32_t key = __float_as_uint(rl[i]) & 0x7FFFFFFFu;
        if ((key & mask) == prefix) b = (key >> shift) & (uint32_t)(nb - 1);
      }
      hist_add_peeled(s_hist, b, lane);
    }
    uint32_t bin, rib;
    (void)find_rank<NT>(s_hist, nb, k_rem, s_wt, s_sel, bin, rib);  // the passes keep at least k_rem entries
    prefix |= bin << shift;
    mask |= (uint32_t)(nb - 1) << shift;
    k_rem = rib;
  }
  const uint32_t T = prefix, rtake = k_rem;
  uint32_t gb = 0, eb = 0;  // keys above T and equal to T before the current block of NT elements
  for (int64_t base = 0; base < sd.d; base += NT) {
    const int64_t i = base + tid;
    uint32_t bits = 0u, fg = 0u, fe = 0u;
    if (i < sd.d) {
      bits = __float_as_uint(rl[i]);
      const uint32_t key = bits & 0x7FFFFFFFu;
      fg = key > T;
      fe = key == T;
    }
    const uint32_t packed = fg | (fe << 16);
    uint32_t tot;
    const uint32_t excl = block_incl_scan<NT>(packed, s_wt, tot) - packed;
    const uint32_t g0 = gb + (excl & 0xFFFFu), e0 = eb + (excl >> 16);
    const uint32_t pos = g0 + (e0 < rtake ? e0 : rtake);
    if ((fg || (fe && e0 < rtake)) && pos < (uint32_t)sd.k) {
      oi[pos] = (int32_t)i;
      ov[pos] = __uint_as_float(bits);
      rl[i] = 0.0f;
    }
    gb += tot & 0xFFFFu;
    eb += tot >> 16;
  }
}

// Appends a layer's dense tiles to the work list of the multi-pass kernels.
template <int NT>
__device__ __forceinline__ void append_tiles(const LargeSeg& ls, uint32_t* __restrict__ counter,
                                             int32_t* __restrict__ items, uint32_t* s_base) {
  const int nt = ls.tile_end - ls.tile_begin;
  __syncthreads();
  if (threadIdx.x == 0) *s_base = atomicAdd(counter, (uint32_t)nt);
  __syncthreads();
  const uint32_t b = *s_base;
  for (int j = threadIdx.x; j < nt; j += NT) items[b + j] = ls.tile_begin + j;
}

// A rejected guess: the early zeros are undone and the layer is selected from the acc values
// in the residual buffer, by the multi-pass kernels if they are enqueued in this call (chain),
// else by this workgroup.  The context's pinned host word is set so that later calls enqueue them.
template <int NT>
__device__ __forceinline__ void reject_layer(int li, const LargeSeg& ls, const SegDesc& sd, uint32_t t_zero,
                                             const uint32_t* __restrict__ chunk_cnt,
                                             const uint2* __restrict__ slots, int nslot, int chain,
                                             LState* __restrict__ lstate, uint32_t* __restrict__ fail_flag,
                                             uint32_t* __restrict__ counter, int32_t* __restrict__ items,
                                             float* __restrict__ res, int32_t* __restrict__ out_idx,
                                             float* __restrict__ out_val, uint32_t* s_hist, uint32_t* s_wt,
                                             uint32_t* s_sel) {
  if (threadIdx.x == 0) {
    lstate[li].mode = MODE_DENSE;
    lstate[li].route = 2u;
    __hip_atomic_store(fail_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  }
  restore_layer<NT>(ls, sd, t_zero, chunk_cnt, slots, nslot, res);
  if (chain) append_tiles<NT>(ls, counter, items, s_sel);
  else rescue_layer<NT>(sd, res, out_idx, out_val, s_hist, s_wt, s_sel);
}

// Partial bucket counts of the layers finished by groups: one workgroup per kCountTiles tiles
// writes its 4096 counts, their sums over runs of 64 buckets, and its totals (candidates,
// candidates at or above tau_top, whether a tile overflowed).  No atomics: k_finish adds the parts.
__global__ __launch_bounds__(1024) void k_group_h(const GroupDesc* __restrict__ hparts,
                                                  const LargeSeg* __restrict__ lsegs,
                                                  const LState* __restrict__ lstate,
                                                  const uint32_t* __restrict__ chunk_cnt,
                                                  const uint2* __restrict__ slots, int nslot,
                                                  uint32_t* __restrict__ bh_part, uint32_t* __restrict__ coarse_part,
                                                  uint4* __restrict__ part_info) {
  constexpr int NW = 16;
  __shared__ uint32_t s_fine[kFineBins];
  __shared__ uint32_t s_tot[3 * NW];
  const GroupDesc hp = hparts[blockIdx.x];
  const LargeSeg ls = lsegs[hp.lseg];
  const LState st = lstate[hp.lseg];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  reinterpret_cast<uint4*>(s_fine)[tid] = make_uint4(0u, 0u, 0u, 0u);
  __syncthreads();
  constexpr int kWcPerPart = kCountTiles / kWaveTiles;
  const int nwc = (ls.chunk_end - ls.chunk_begin + kWaveTiles - 1) / kWaveTiles;
  const int q_end = (hp.first + 1) * kWcPerPart < nwc ? (hp.first + 1) * kWcPerPart : nwc;
  uint32_t n = 0, n_top = 0, over = 0;  // wave-uniform
  for (int q = hp.first * kWcPerPart + w; q < q_end; q += NW) {
    const int c0 = ls.chunk_begin + q * kWaveTiles;
    const uint32_t raw = (lane < kWaveTiles && c0 + lane < ls.chunk_end) ? chunk_cnt[c0 + lane] : 0u;
    over |= __ballot(raw > (uint32_t)nslot) != 0ull;
    n += wave_sum(raw);
    const WaveChunk wc = wc_open(c0, ls.chunk_end, chunk_cnt, nslot, lane);
    n_top += wc_count(wc, slots, nslot, st.tau, st.tau_top, st.shift, s_fine, lane);
  }
  if (lane == 0) { s_tot[w] = n; s_tot[NW + w] = n_top; s_tot[2 * NW + w] = over; }
  __syncthreads();
  const uint4 mine = reinterpret_cast<const uint4*>(s_fine)[tid];
  reinterpret_cast<uint4*>(bh_part + (int64_t)blockIdx.x * kFineBins)[tid] = mine;
  // buckets 64 c .. 64 c + 63 are held by the 16 threads 16 c .. 16 c + 15
  uint32_t c4 = (mine.x + mine.y) + (mine.z + mine.w);
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) c4 += __shfl_xor(c4, o, 64);
  if ((tid & 15) == 0) coarse_part[(int64_t)blockIdx.x * kCoarseBins + (tid >> 4)] = c4;
  if (tid == 0) {
    uint4 info = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int i = 0; i < NW; ++i) { info.x += s_tot[i]; info.y += s_tot[NW + i]; info.z |= s_tot[2 * NW + i]; }
    part_info[blockIdx.x] = info;
  }
}

// Among 64 counts c[0..63] held one per lane (ordered by key), the bin that holds the entry of
// rank `rank` counted from bin 63 downwards, and the rank inside that bin; false if they hold
// fewer than `rank`.  Wave-uniform result.
__device__ __forceinline__ bool wave_find_rank64(uint32_t c, uint32_t rank, int lane, uint32_t& bin,
                                                 uint32_t& rank_in_bin, uint32_t& count_in_bin) {
  const uint32_t rev = __shfl(c, 63 - lane, 64);           // lane l holds bin 63 - l
  const uint32_t incl = wave_incl_scan(rev, lane);         // entries in bins 63 - l .. 63
  const uint64_t reach = __ballot(incl >= rank);
  if (reach == 0ull) return false;
  const int l = __builtin_ctzll(reach);
  const uint32_t at = (uint32_t)__builtin_amdgcn_readlane((int)incl, l), own = (uint32_t)__builtin_amdgcn_readlane((int)rev, l);
  bin = (uint32_t)(63 - l);
  rank_in_bin = rank - (at - own);
  count_in_bin = own;
  return true;
}

// One workgroup per large layer.  Layers that are not sampled hand their tiles to the
// multi-pass kernels.  Sampled layers get their verdict and decisive bucket; those of at most
// kFusedTiles tiles are finished here, the others by k_group_a and k_group_b.
// Two launches share the layers (`list` holds the launch's large-layer indices): workgroups of
// 256 threads take the sampled layers of at most kFinishSmallTiles tiles that one workgroup
// finishes, workgroups of 1024 threads all others.  A CU holds six of the small workgroups side
// by side, against two of the large ones.
template <int NT>
__global__ __launch_bounds__(NT) void k_finish(const int32_t* __restrict__ list,
                                               const SegDesc* __restrict__ segs,
                                                 const LargeSeg* __restrict__ lsegs,
                                                 LState* __restrict__ lstate,
                                                 const uint32_t* __restrict__ chunk_cnt,
                                                 const uint2* __restrict__ slots, int nslot,
                                                 const uint32_t* __restrict__ bh_part,
                                                 const uint32_t* __restrict__ coarse_part,
                                                 const uint4* __restrict__ part_info,
                                                 float* __restrict__ res, int32_t* __restrict__ out_idx,
                                                 float* __restrict__ out_val, uint32_t* __restrict__ counter,
                                                 int32_t* __restrict__ items, int chain,
                                                 uint32_t* __restrict__ fail_flag) {
  constexpr int NW = NT / 64;
  constexpr int kMaxWc = kFusedTiles / kWaveTiles;
  static_assert(kMaxWc <= NT, "one thread per wave chunk in the scan of their counts");
  static_assert(NT == 256 || NT == 1024, "the two launches");
  static_assert(kFinishSmallTiles <= 256 / 64 * kWaveChunks * kWaveTiles &&
                    kFusedTiles <= 1024 / 64 * kWaveChunks * kWaveTiles,
                "a wave walks at most kWaveChunks wave chunks");
  // the small workgroups keep a shorter band: with 24 KB of LDS a CU holds six of them
  constexpr int BAND = NT == 256 ? kBandCapSmall : kBandCap;
  __shared__ uint2 s_band[BAND];
  __shared__ uint32_t s_fine[kFineBins];   // bucket counts; the rescue's histograms reuse it
  __shared__ uint32_t s_wt[2 * NW];
  __shared__ uint32_t s_sel[2];
  __shared__ uint32_t s_ti[2];
  __shared__ uint32_t s_nband;
  __shared__ uint32_t s_wgt[kMaxWc];
  static_assert(kFineBins >= kBins0, "the rescue's histogram fits");
  const int li = list[blockIdx.x], tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const LargeSeg ls = lsegs[li];
  if (finish_small(ls) != (NT == 256)) return;  // never: the host's lists follow the same rule
  const SegDesc sd = segs[ls.seg];
  if (!ls.sampled) {  // uniform over the workgroup
    append_tiles<NT>(ls, counter, items, s_sel);
    return;
  }
  const LState st = lstate[li];
  const int nwc = (ls.chunk_end - ls.chunk_begin + kWaveTiles - 1) / kWaveTiles;
  const uint32_t k = (uint32_t)sd.k;
  uint32_t n = 0, ntop = 0, bstar = 0, k_rem = 0, n_band = 0;
  int over = 0;
  bool ok;  // uniform over the workgroup
  WaveChunk wcs[kWaveChunks];  // wave w walks the wave chunks w, w + NW, ... of a layer finished here
  WaveEntries we;
  if (ls.fused) {
    // totals of the tiles (candidates, overflowed tiles) and bucket counts of the own slots
    for (int c = ls.chunk_begin + tid; c < ls.chunk_end; c += NT) {  // at most kFusedTiles <= NT tiles
      const uint32_t v = chunk_cnt[c];
      over |= v > (uint32_t)nslot;
      n += v;
    }
    for (int i = tid; i < kFineBins / 4; i += NT) reinterpret_cast<uint4*>(s_fine)[i] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kWaveChunks; ++i)  // a chunk that starts at or after chunk_end is empty
      wcs[i] = wc_open(ls.chunk_begin + (w + i * NW) * kWaveTiles, ls.chunk_end, chunk_cnt, nslot, lane);
    wc_load4(wcs, slots, nslot, lane, we);
    wc_for_each4(wcs, we, slots, nslot, lane, [&](int, uint2 en, bool live) {
      entry_count(en, live, st.tau, st.tau_top, st.shift, s_fine, ntop);
    });
    ntop = lane == 0 ? ntop : 0u;  // the count is wave-uniform: one lane carries it into the sum
    block_sum2<NT>(n, ntop, s_wt);
    over = __syncthreads_or(over);
    ok = !over && n >= k && ntop < k;
    if (ok) {
      ok = find_rank<NT>(s_fine, kFineBins, k - ntop, s_wt, s_sel, bstar, k_rem);
      if (ok) n_band = s_fine[bstar];
    }
  } else {
    // the parts that k_group_h wrote: totals, then the run of 64 buckets that holds the k-th
    // largest key from the coarse counts, then the bucket inside that run
    const int h0 = ls.group_h_begin, np = ls.group_h_end - ls.group_h_begin;
    for (int h = tid; h < np; h += NT) {
      const uint4 info = part_info[h0 + h];
      n += info.x;
      ntop += info.y;
      over |= info.z != 0u;
    }
    block_sum2<NT>(n, ntop, s_wt);
    over = __syncthreads_or(over);
    ok = !over && n >= k && ntop < k;
    if (ok) {  // wave w adds the parts w, w + 16, ...; every wave then adds the 16 rows for itself
      static_assert(kCoarseBins == 64 && kFineBins == 64 * kCoarseBins, "one lane per bin at both levels");
      uint32_t acc = 0;
      for (int h = w; h < np; h += 4 * NW) {
        uint32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          v[u] = h + u * NW < np ? coarse_part[(int64_t)(h0 + h + u * NW) * kCoarseBins + lane] : 0u;
        acc += (v[0] + v[1]) + (v[2] + v[3]);
      }
      s_fine[w * 64 + lane] = acc;
      __syncthreads();
      uint32_t c = 0;
#pragma unroll
      for (int i = 0; i < NW; ++i) c += s_fine[i * 64 + lane];
      uint32_t crun = 0, rank_in_run = 0, unused = 0;
      ok = wave_find_rank64(c, k - ntop, lane, crun, rank_in_run, unused);
      __syncthreads();
      if (ok) {
        acc = 0;
        for (int h = w; h < np; h += 4 * NW) {
          uint32_t v[4];
#pragma unroll
          for (int u = 0; u < 4; ++u)
            v[u] = h + u * NW < np ? bh_part[(int64_t)(h0 + h + u * NW) * kFineBins + crun * 64u + lane] : 0u;
          acc += (v[0] + v[1]) + (v[2] + v[3]);
        }
        s_fine[w * 64 + lane] = acc;
        __syncthreads();
        c = 0;
#pragma unroll
        for (int i = 0; i < NW; ++i) c += s_fine[i * 64 + lane];
        uint32_t b = 0;
        ok = wave_find_rank64(c, rank_in_run, lane, b, k_rem, n_band);
        bstar = crun * 64u + b;
      }
    }
  }
  ok = ok && n_band <= (uint32_t)BAND;
  if (!ok) {
    reject_layer<NT>(li, ls, sd, st.t_zero, chunk_cnt, slots, nslot, chain, lstate, fail_flag, counter, items, res,
                     out_idx, out_val, s_fine, s_wt, s_sel);
    return;
  }
  if (!ls.fused) {
    if (tid == 0) {
      lstate[li].mode = MODE_SPARSE;
      lstate[li].bstar = bstar;
      lstate[li].k_rem = k_rem;
      lstate[li].n_band = n_band;
    }
    return;
  }
  // one workgroup finishes the layer: a wave takes every 16th wave chunk
  if (tid == 0) s_nband = 0u;
  __syncthreads();
  {
    uint32_t n_gt[kWaveChunks] = {0u, 0u, 0u, 0u};
    wc_for_each4(wcs, we, slots, nslot, lane, [&](int i, uint2 en, bool live) {
      entry_phase_a(en, live, st.tau, st.tau_top, st.shift, bstar, s_band, BAND, &s_nband, n_gt[i]);
    });
#pragma unroll
    for (int i = 0; i < kWaveChunks; ++i)
      if (lane == 0 && w + i * NW < nwc) s_wgt[w + i * NW] = n_gt[i];
  }
  __syncthreads();
  const uint32_t m = s_nband < (uint32_t)BAND ? s_nband : (uint32_t)BAND;  // equals n_band
  if (tid == 0) { s_ti[0] = 0xFFFFFFFFu; s_ti[1] = 0u; }
  // exclusive scan of the wave chunks' counts (in place)
  {
    const uint32_t v = tid < nwc ? s_wgt[tid] : 0u;
    uint32_t tot;
    const uint32_t incl = block_incl_scan<NT>(v, s_wt, tot);
    if (tid < nwc) s_wgt[tid] = incl - v;
  }
  __syncthreads();
  band_select<NT>(s_band, m, k_rem, st.tau + (bstar << st.shift), st.shift, s_fine, s_wt, s_sel, s_ti);
  const uint32_t T = s_ti[0], I = s_ti[1];
  int32_t* oi = out_idx + sd.out_offset;
  float* ov = out_val + sd.out_offset;
  float* rl = res + sd.offset;
  {
    // a chunk's first output position: the candidates above b* and the kept band entries before it
    uint32_t pos[kWaveChunks];
#pragma unroll
    for (int i = 0; i < kWaveChunks; ++i) {
      const int q = w + i * NW;
      pos[i] = 0u;
      if (q < nwc)  // wave-uniform
        pos[i] = s_wgt[q] + band_kept_before(s_band, m, T, I, (uint32_t)q * (uint32_t)(kWaveTiles * kTile), lane);
    }
    wc_for_each4(wcs, we, slots, nslot, lane, [&](int i, uint2 en, bool live) {
      entry_phase_b(en, live, T, I, st.t_zero, pos[i], k, sd.d, oi, ov, rl);
    });
  }
  if (tid == 0) {
    lstate[li].mode = MODE_SPARSE;
    lstate[li].route = 1u;
  }
}

// Phase A of the layers finished by groups: one workgroup per group of 64 tiles, one wave per
// wave chunk.  Writes the wave chunks' counts of candidates above b* and the group's band entries.
__global__ __launch_bounds__(kGroupWaves * 64) void k_group_a(const GroupDesc* __restrict__ groups,
                                                            const LargeSeg* __restrict__ lsegs,
                                                            LState* __restrict__ lstate,
                                                            const uint32_t* __restrict__ chunk_cnt,
                                                            const uint2* __restrict__ slots, int nslot,
                                                            uint32_t* __restrict__ wgt, uint2* __restrict__ band,
                                                            uint32_t* __restrict__ band_cnt) {
  __shared__ uint32_t s_nband;
  const GroupDesc gd = groups[blockIdx.x];
  const LState st = lstate[gd.lseg];
  if (st.mode != MODE_SPARSE) return;  // uniform over the workgroup
  const LargeSeg ls = lsegs[gd.lseg];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  if (tid == 0) s_nband = 0u;
  __syncthreads();
  const int q = gd.first * kGroupWaves + w;  // wave chunk inside the layer
  const int c0 = ls.chunk_begin + q * kWaveTiles;
  if (c0 < ls.chunk_end) {  // wave-uniform
    const WaveChunk wc = wc_open(c0, ls.chunk_end, chunk_cnt, nslot, lane);
    const uint32_t n_gt = wc_phase_a(wc, slots, nslot, st.tau, st.tau_top, st.shift, st.bstar,
                                     band + (int64_t)blockIdx.x * kGroupBand, kGroupBand, &s_nband, lane);
    if (lane == 0) wgt[ls.wchunk_begin + q] = n_gt;
  }
  __syncthreads();
  if (tid == 0) {
    const uint32_t nb = s_nband;
    band_cnt[blockIdx.x] = nb < (uint32_t)kGroupBand ? nb : (uint32_t)kGroupBand;
    if (nb > (uint32_t)kGroupBand) lstate[gd.lseg].band_over = 1u;  // every writer stores the same value
  }
}

// Between the phases of the layers finished by groups: one workgroup per such layer gathers the
// band from all groups, selects T and I, and turns the wave chunks' counts of candidates above
// b* into output positions (exclusive scan of count + kept band entries of the wave chunk, in
// place).  If some group's band overflowed, the layer is selected from the residual buffer instead.
__global__ __launch_bounds__(1024) void k_group_p(const int32_t* __restrict__ multi,
                                                  const SegDesc* __restrict__ segs,
                                                  const LargeSeg* __restrict__ lsegs,
                                                  LState* __restrict__ lstate,
                                                  const uint32_t* __restrict__ chunk_cnt,
                                                  const uint2* __restrict__ slots, int nslot,
                                                  uint32_t* __restrict__ wgt,
                                                  const uint2* __restrict__ band,
                                                  const uint32_t* __restrict__ band_cnt,
                                                  float* __restrict__ res, int32_t* __restrict__ out_idx,
                                                  float* __restrict__ out_val, uint32_t* __restrict__ counter,
                                                  int32_t* __restrict__ items, int chain,
                                                  uint32_t* __restrict__ fail_flag) {
  constexpr int NT = 1024;
  __shared__ uint2 s_band[kBandCap];
  __shared__ uint32_t s_hist[4 * NT];   // rescue histogram / group offsets / sub-buckets / kept band entries per wave chunk
  __shared__ uint32_t s_wt[32];
  __shared__ uint32_t s_sel[2];
  __shared__ uint32_t s_ti[2];
  static_assert(4 * NT >= kBins0, "the rescue's histogram fits");
  const int tid = threadIdx.x;
  const int li = multi[blockIdx.x];
  const LState st = lstate[li];
  if (st.mode != MODE_SPARSE) return;  // rejected by k_finish, dealt with there
  const LargeSeg ls = lsegs[li];
  if (st.band_over) {  // uniform over the workgroup
    reject_layer<NT>(li, ls, segs[ls.seg], st.t_zero, chunk_cnt, slots, nslot, chain, lstate, fail_flag, counter,
                     items, res, out_idx, out_val, s_hist, s_wt, s_sel);
    return;
  }
  // the counts of the first 4096 wave chunks are loaded now and used at the end (the plan aligns
  // a layer's first wave chunk to 4 entries, and pads its last group of 4)
  const int nwc = (ls.chunk_end - ls.chunk_begin + kWaveTiles - 1) / kWaveTiles;
  uint4* wl4 = reinterpret_cast<uint4*>(wgt + ls.wchunk_begin);
  uint4 first = make_uint4(0u, 0u, 0u, 0u);
  if (4 * tid < nwc) first = wl4[tid];
  // the layer's band: the groups' entries one after the other (any order serves the selection);
  // thread e copies entry e, its group found by a search over the groups' offsets
  uint32_t m = 0;
  uint32_t* s_off = s_hist;  // NT words
  for (int g0 = ls.group_begin; g0 < ls.group_end; g0 += NT) {  // uniform trip count
    const int g = g0 + tid;
    const uint32_t cnt = g < ls.group_end ? band_cnt[g] : 0u;
    uint32_t tot;
    s_off[tid] = block_incl_scan<NT>(cnt, s_wt, tot) - cnt;
    __syncthreads();
    for (uint32_t e = tid; e < tot; e += NT) {
      int lo = 0, hi = NT - 1;  // last group whose offset is <= e
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (s_off[mid] <= e) lo = mid; else hi = mid - 1;
      }
      const uint32_t i = e - s_off[lo];
      if (m + e < (uint32_t)kBandCap && i < (uint32_t)kGroupBand) s_band[m + e] = band[(int64_t)(g0 + lo) * kGroupBand + i];
    }
    m += tot;
    __syncthreads();
  }
  m = m < (uint32_t)kBandCap ? m : (uint32_t)kBandCap;  // equals n_band
  if (tid == 0) { s_ti[0] = 0xFFFFFFFFu; s_ti[1] = 0u; }
  __syncthreads();
  band_select<NT>(s_band, m, st.k_rem, st.tau + (st.bstar << st.shift), st.shift, s_hist, s_wt, s_sel, s_ti);
  const uint32_t T = s_ti[0], I = s_ti[1];
  // output position of every wave chunk's first kept entry: exclusive scan of (count above b* +
  // kept band entries of the wave chunk), 4096 wave chunks per round, four per thread
  uint32_t* s_blk = s_hist;  // 4 * NT words
  uint32_t carry = 0;
  for (int base = 0; base < nwc; base += 4 * NT) {  // uniform trip count
    __syncthreads();
    reinterpret_cast<uint4*>(s_blk)[tid] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();
    for (uint32_t i = tid; i < m; i += NT) {
      const uint2 en = s_band[i];
      const uint32_t key = en.y & 0x7FFFFFFFu;
      const uint32_t q = en.x / (uint32_t)(kWaveTiles * kTile) - (uint32_t)base;  // wraps to a large value below base
      if ((key > T || (key == T && en.x <= I)) && q < (uint32_t)(4 * NT)) atomicAdd(&s_blk[q], 1u);
    }
    __syncthreads();
    const bool in = base + 4 * tid < nwc;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (in) v = base == 0 ? first : wl4[base / 4 + tid];
    const uint4 bk = reinterpret_cast<const uint4*>(s_blk)[tid];
    v.x += bk.x; v.y += bk.y; v.z += bk.z; v.w += bk.w;   // entries past the layer's last wave chunk are padding
    const uint32_t sum = (v.x + v.y) + (v.z + v.w);
    uint32_t tot;
    const uint32_t excl = carry + block_incl_scan<NT>(sum, s_wt, tot) - sum;
    if (in) wl4[base / 4 + tid] = make_uint4(excl, excl + v.x, excl + v.x + v.y, excl + v.x + v.y + v.z);
    carry += tot;
  }
  if (tid == 0) {
    lstate[li].T = T;
    lstate[li].I = I;
    lstate[li].route = 1u;
  }
}

// Phase B of the layers finished by groups: one workgroup per group, one wave per wave chunk,
// which emits its kept entries from the position that k_group_p computed.
__global__ __launch_bounds__(kGroupWaves * 64) void k_group_b(const GroupDesc* __restrict__ groups,
                                                            const SegDesc* __restrict__ segs,
                                                            const LargeSeg* __restrict__ lsegs,
                                                            const LState* __restrict__ lstate,
                                                            const uint32_t* __restrict__ chunk_cnt,
                                                            const uint2* __restrict__ slots, int nslot,
                                                            const uint32_t* __restrict__ wgt,
                                                            float* __restrict__ res, int32_t* __restrict__ out_idx,
                                                            float* __restrict__ out_val) {
  const GroupDesc gd = groups[blockIdx.x];
  const LState st = lstate[gd.lseg];
  if (st.mode != MODE_SPARSE || st.band_over) return;  // uniform over the workgroup
  const LargeSeg ls = lsegs[gd.lseg];
  const SegDesc sd = segs[ls.seg];
  const int lane = lane_id(), w = threadIdx.x >> 6;
  const int q = gd.first * kGroupWaves + w;
  const int c0 = ls.chunk_begin + q * kWaveTiles;
  if (c0 >= ls.chunk_end) return;  // wave-uniform
  const uint32_t pos0 = wgt[ls.wchunk_begin + q];
  const WaveChunk wc = wc_open(c0, ls.chunk_end, chunk_cnt, nslot, lane);
  wc_phase_b(wc, slots, nslot, st.T, st.I, st.t_zero, pos0, (uint32_t)sd.k, sd.d, out_idx + sd.out_offset,
             out_val + sd.out_offset, res + sd.offset, lane);
}

// ------------------------------------------------------------------ multi-pass select
// Radix select over the acc values in the residual buffer, multi-block: layers that are not
// sampled, and layers whose guess was rejected when these kernels are enqueued.  The tiles
// come from the device-built work list `items`; kDenseGrid workgroups stride over it.
struct TileWork {
  float* res;          // the tile's residual data
  int n;               // valid entries
  int lseg;
  int local0;          // layer-local index of the first element
  int slot;            // index into tile_gt / tile_eq
  bool skip_level0;    // level-0 histogram already made by the streaming pass
};

__device__ __forceinline__ void get_tile(int item, const TileDesc* __restrict__ tiles,
                                         const int32_t* __restrict__ items, float* res, TileWork& tw) {
  const int t = items[item];
  const TileDesc td = tiles[t];
  tw.lseg = td.seg;
  tw.slot = t;
  tw.local0 = td.local0;
  tw.res = res + td.start;
  tw.n = td.n;
  tw.skip_level0 = td.ctile < 0;
}

__device__ __forceinline__ void load_tile(const TileWork& tw, int w, int lane, uint32_t (&a)[kTileV][4]) {
  const int n_w = tw.n - w * kWaveChunk;
  const float* r = tw.res + w * kWaveChunk;
  load_bits<kTileV>(r, n_w, aligned16(r, r), lane, a);
}

// One digit of the radix select, decided from the layer's histogram of that digit (complete
// since the previous launch): every workgroup that needs the result computes it for itself,
// and the workgroup that holds the layer's first tile also records it in the layer's state for
// the launches after this one.  k_before: entries still to take before this digit.
// Returns false if the histogram holds fewer than k_before entries (nothing to select).
__device__ __forceinline__ bool decide_digit(const uint32_t* __restrict__ gh, int nb, int shift, uint32_t p_before,
                                             uint32_t k_before, uint32_t* s_wt, uint32_t* s_sel,
                                             uint32_t& p_after, uint32_t& k_after) {
  uint32_t bin;
  const bool found = find_rank<256>(gh, nb, k_before, s_wt, s_sel, bin, k_after);
  p_after = p_before | (bin << shift);
  return found;
}

// Histogram of one radix digit over the entries whose higher key bits equal the prefix
// (levels 1 and 2 first decide the digit before theirs from its histogram).
template <int LEVEL>
__global__ __launch_bounds__(256) void k_hist(const TileDesc* __restrict__ tiles,
                                              const int32_t* __restrict__ items,
                                              const uint32_t* __restrict__ counter,
                                              const LargeSeg* __restrict__ lsegs,
                                              const SegDesc* __restrict__ segs,
                                              float* __restrict__ res,
                                              DState* __restrict__ dstate,
                                              uint32_t* __restrict__ ghist) {
  __shared__ uint32_t s_hist[LEVEL == 0 ? kBins0 : kBins12];
  __shared__ uint32_t s_wt[4];
  __shared__ uint32_t s_sel[2];
  constexpr int shift = LEVEL == 0 ? 20 : (LEVEL == 1 ? 10 : 0);
  constexpr uint32_t mask = LEVEL == 0 ? 0u : (LEVEL == 1 ? 0x7FF00000u : 0x7FFFFC00u);
  constexpr int nb = LEVEL == 0 ? kBins0 : kBins12;
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const int end = (int)*counter;
  for (int item = blockIdx.x; item < end; item += kDenseGrid) {
    TileWork tw;
    get_tile(item, tiles, items, res, tw);
    if (LEVEL == 0 && tw.skip_level0) continue;
    uint32_t* gh = ghist + (int64_t)tw.lseg * kHistStride;
    uint32_t prefix = 0u;
    if (LEVEL == 1) {
      uint32_t kr;
      if (!decide_digit(gh, kBins0, 20, 0u, (uint32_t)segs[lsegs[tw.lseg].seg].k, s_wt, s_sel, prefix, kr)) continue;
      if (tw.local0 == 0 && tid == 0) { dstate[tw.lseg].p0 = prefix; dstate[tw.lseg].k0 = kr; }
    } else if (LEVEL == 2) {
      uint32_t kr;
      const uint32_t p0 = dstate[tw.lseg].p0, k0 = dstate[tw.lseg].k0;
      if (!decide_digit(gh + kHistLevel1, kBins12, 10, p0, k0, s_wt, s_sel, prefix, kr)) continue;
      if (tw.local0 == 0 && tid == 0) { dstate[tw.lseg].p1 = prefix; dstate[tw.lseg].k1 = kr; }
    }
    __syncthreads();
    for (int i = tid; i < nb; i += 256) s_hist[i] = 0u;
    uint32_t a[kTileV][4];
    load_tile(tw, w, lane, a);
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

// Decides the last digit (which fixes the k-th largest key T and the number of entries equal
// to T to take), then counts per tile how many keys are above T and how many equal T.
__global__ __launch_bounds__(256) void k_count(const TileDesc* __restrict__ tiles,
                                               const int32_t* __restrict__ items,
                                               const uint32_t* __restrict__ counter,
                                               float* __restrict__ res,
                                               DState* __restrict__ dstate,
                                               const uint32_t* __restrict__ ghist,
                                               uint32_t* __restrict__ tile_gt,
                                               uint32_t* __restrict__ tile_eq) {
  __shared__ uint32_t s_g[4], s_e[4];
  __shared__ uint32_t s_wt[4];
  __shared__ uint32_t s_sel[2];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const int end = (int)*counter;
  for (int item = blockIdx.x; item < end; item += kDenseGrid) {
    TileWork tw;
    get_tile(item, tiles, items, res, tw);
    uint32_t T, rtake;
    const uint32_t p1 = dstate[tw.lseg].p1, k1 = dstate[tw.lseg].k1;
    if (!decide_digit(ghist + (int64_t)tw.lseg * kHistStride + kHistLevel2, kBins12, 0, p1, k1, s_wt, s_sel, T,
                      rtake))
      continue;
    if (tw.local0 == 0 && tid == 0) { dstate[tw.lseg].prefix = T; dstate[tw.lseg].k_rem = rtake; }
    uint32_t a[kTileV][4];
    load_tile(tw, w, lane, a);
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

// Exclusive scan of the per-tile counts inside each large layer that takes the multi-pass
// route (in place).
__global__ __launch_bounds__(1024) void k_scan(const LargeSeg* __restrict__ lsegs,
                                               const LState* __restrict__ lstate,
                                               uint32_t* __restrict__ tile_gt,
                                               uint32_t* __restrict__ tile_eq) {
  __shared__ uint32_t s_wt[16];
  const LargeSeg ls = lsegs[blockIdx.x];
  if (lstate[blockIdx.x].mode != MODE_DENSE) return;
  const int begin = ls.tile_begin, end = ls.tile_end;
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
__global__ __launch_bounds__(256) void k_emit(const TileDesc* __restrict__ tiles,
                                              const int32_t* __restrict__ items,
                                              const uint32_t* __restrict__ counter,
                                              const LargeSeg* __restrict__ lsegs,
                                              const SegDesc* __restrict__ segs,
                                              float* __restrict__ res,
                                              const DState* __restrict__ dstate,
                                              const uint32_t* __restrict__ tile_gt,
                                              const uint32_t* __restrict__ tile_eq,
                                              int32_t* __restrict__ out_idx,
                                              float* __restrict__ out_val) {
  __shared__ uint32_t s_g[4], s_e[4];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const int end = (int)*counter;
  for (int item = blockIdx.x; item < end; item += kDenseGrid) {
    TileWork tw;
    get_tile(item, tiles, items, res, tw);
    const DState st = dstate[tw.lseg];
    const uint32_t T = st.prefix, rtake = st.k_rem;
    const uint32_t tg = tile_gt[tw.slot], te = tile_eq[tw.slot];
    const SegDesc sd = segs[lsegs[tw.lseg].seg];
    const int n_w = tw.n - w * kWaveChunk;
    uint32_t a[kTileV][4];
    load_tile(tw, w, lane, a);
    uint32_t cg, ce;
    lane_count<kTileV>(a, n_w, lane, T, cg, ce);
    cg = wave_sum(cg);
    ce = wave_sum(ce);
    __syncthreads();
    if (lane == 0) { s_g[w] = cg; s_e[w] = ce; }
    __syncthreads();
    uint32_t gb = tg, eb = te;
    for (int i = 0; i < w; ++i) { gb += s_g[i]; eb += s_e[i]; }
    // nothing to emit in this wave if it holds no key above T and its ties come too late
    if (cg == 0 && (ce == 0 || eb >= rtake)) continue;
    float* r = tw.res + w * kWaveChunk;
    wave_emit<kTileV, EMIT_ZERO>(a, n_w, lane, T, rtake, gb, eb, (uint32_t)sd.k, tw.local0 + w * kWaveChunk,
                                 out_idx + sd.out_offset, out_val + sd.out_offset, r, aligned16(r, r));
  }
}

// ------------------------------------------------------------------ merge ----
// Algorithm 1 lines 8-9.  Two kernels.
//
// k_merge_bounds: for every worker and layer, where each 8192-element tile of the dense
// update starts in the worker's sorted index list: bounds[slot0 + t][p] = first list position
// whose index lies in tile t or later; bounds[slot0 + ntiles][p] = k.  One pass over the lists.
__global__ __launch_bounds__(256) void k_merge_bounds(const BChunk* __restrict__ chunks,
                                                      const SegDesc* __restrict__ segs,
                                                      const int32_t* __restrict__ idx, int64_t stride_k,
                                                      int nb, int32_t* __restrict__ bounds) {
  constexpr int U = kBoundChunk / 256;
  const BChunk bc = chunks[blockIdx.x];
  const int p = blockIdx.y;
  const SegDesc sd = segs[bc.seg];
  const int32_t* li = idx + (int64_t)p * stride_k + sd.out_offset;
  // slot-major layout: the P workers' entries of one tile slot are adjacent, so a merge
  // workgroup reads all its workers' bounds from one or two cache lines
  const int P = gridDim.y;
  int32_t* b = bounds + (int64_t)bc.slot0 * P + p;
  const int jend = sd.k < bc.j0 + kBoundChunk ? sd.k : bc.j0 + kBoundChunk;
  // all loads of the thread first (an entry and its predecessor), then the stores
  int cur[U], prev[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int j = bc.j0 + u * 256 + (int)threadIdx.x;
    cur[u] = j < jend ? li[j] : 0;
    prev[u] = (j < jend && j > 0) ? li[j - 1] : 0;
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int j = bc.j0 + u * 256 + (int)threadIdx.x;
    if (j >= jend) continue;
    // indices are clamped into the layer so that bad input cannot write outside the row
    const int i1 = cur[u] < 0 ? 0 : (cur[u] >= sd.d ? sd.d - 1 : cur[u]);
    const int t = i1 / kMergeTile;
    int tp = -1;
    if (j > 0) {
      const int i0 = prev[u] < 0 ? 0 : (prev[u] >= sd.d ? sd.d - 1 : prev[u]);
      tp = i0 / kMergeTile;
    }
    for (int q = tp + 1; q <= t; ++q) b[(int64_t)q * P] = j;
    if (j == sd.k - 1)
      for (int q = t + 1; q <= bc.ntiles; ++q) b[(int64_t)q * P] = sd.k;
  }
}

// Accumulation shared by the merge-type kernels: the workgroup that owns one tile of the
// dense layout loads the entries of all workers that fall into the tile (found through the
// bounds, no searching) and adds them into the LDS tile s_acc so that every element holds the
// sum of its entries in worker order.
// T = float: binary32 adds, the sum the method defines.  T = double: exact-order double sums for
// the delta metric.
//
// Order only matters for an element that three or more workers selected: 0 + a + b is the same
// binary32 value in either order (0 + x is x, or +0 for x = -0, and the sum of two values is
// commutative).  So the float accumulation adds all entries at once (compare-and-swap on the
// element's bits with a correctly rounded add), while three bitmaps record which elements were
// hit once, twice and three times.  The elements hit three times or more (none in most tiles
// when the workers together keep about 1 % of the layer, a handful when they keep 10 %) are
// repaired afterwards: their entries are collected in a short LDS list and one thread per such
// element adds them again in worker order.  Tiles with more than 1024 entries (the entries no
// longer fit the registers of one pass), a list that overflows, and more than 256 workers take
// the plain way: one barrier per worker (inside one worker the indices are distinct).
// s_multi: kMergeMultiWords words (float only).  merge_accumulate returns the number of entries
// that fell into the tile.
constexpr int kMergeBitWords = kMergeTile / 32;          // words of one bitmap
constexpr int kMergeRepairCap = kMergeBitWords;          // list entries: they reuse the first two bitmaps (8 bytes each)
constexpr int kMergeMultiWords = 3 * kMergeBitWords + 2; // once, twice, thrice, [flag], [list count]

// Entry table of one batch of up to 256 workers for one tile: s_start[q] = number of entries of
// the workers before q that fall into the tile, s_start[256] = their total (returned), s_lo[q] =
// where worker q's entries start in its list.  Ends with a barrier.
__device__ __forceinline__ uint32_t merge_table(uint32_t* s_start, int32_t* s_lo, uint32_t* s_wt, int32_t k,
                                                int slot, int p0, int np, int P,
                                                const int32_t* __restrict__ bounds) {
  const int tid = threadIdx.x;
  int lo = 0;
  uint32_t cnt = 0;
  if (tid < np) {
    const int32_t* b = bounds + (int64_t)slot * P + (p0 + tid);  // slot-major: adjacent workers, adjacent words
    int hi = b[P];
    lo = b[0];
    lo = lo < 0 ? 0 : (lo > k ? k : lo);
    hi = hi < 0 ? 0 : (hi > k ? k : hi);
    cnt = hi > lo ? (uint32_t)(hi - lo) : 0u;
  }
  uint32_t total;
  const uint32_t incl = block_incl_scan<256>(cnt, s_wt, total);
  s_start[tid] = incl - cnt;
  s_lo[tid] = lo;
  if (tid == 0) s_start[256] = total;
  __syncthreads();
  return total;
}

// Entry e of the batch's table: its worker q (-1 if e >= total), offset inside the tile and value.
__device__ __forceinline__ void merge_entry(uint32_t e, uint32_t total, const uint32_t* s_start, const int32_t* s_lo,
                                            const TileDesc& td, const SegDesc& sd, int p0, int np,
                                            const int32_t* __restrict__ idx, const float* __restrict__ val,
                                            int64_t stride_k, int& q, uint32_t& off, float& v) {
  q = -1;
  off = 0xFFFFFFFFu;
  v = 0.f;
  if (e < total) {
    int a = 0, z = np;  // last worker q with s_start[q] <= e (skips workers without entries here)
    while (a < z) {
      const int mid = (a + z) >> 1;
      if (s_start[mid] <= e) a = mid + 1; else z = mid;
    }
    q = a - 1;
    const int64_t gi = (int64_t)(p0 + q) * stride_k + sd.out_offset + s_lo[q] + (int)(e - s_start[q]);
    off = (uint32_t)(idx[gi] - td.local0);
    v = val[gi];
  }
}

// Adds the `total` entries of the batch's table into s_acc in worker order, one barrier per
// worker.  Ends with a barrier.
template <typename T>
__device__ __forceinline__ void merge_entries_ordered(T* s_acc, const uint32_t* s_start, const int32_t* s_lo,
                                                      uint32_t total, const TileDesc& td, const SegDesc& sd, int p0,
                                                      int np, const int32_t* __restrict__ idx,
                                                      const float* __restrict__ val, int64_t stride_k) {
  const int tid = threadIdx.x;
  for (uint32_t base = 0; base < total; base += 1024) {
    int pe[4];
    uint32_t off[4];
    float v[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
      merge_entry(base + (uint32_t)(r * 256 + tid), total, s_start, s_lo, td, sd, p0, np, idx, val, stride_k, pe[r],
                  off[r], v[r]);
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

// The unordered accumulation of a tile with at most 1024 entries (four per thread, which stay
// in registers for the repair).  All entries are added at once; then the elements whose bit is
// set in `thrice` get the sum of their entries in worker order: their entries are collected
// (key = offset | worker << 16, value) in the space of the first two bitmaps, and the thread that
// holds an element's first entry adds the element's entries by increasing worker.  Returns false
// (uniform; s_acc is then to be cleared and filled the ordered way) if there are more than
// kMergeRepairCap such entries.  Ends with a barrier.
__device__ __forceinline__ bool merge_entries_unordered(float* s_acc, const uint32_t* s_start, const int32_t* s_lo,
                                                        uint32_t* s_multi, uint32_t total, const TileDesc& td,
                                                        const SegDesc& sd, int np, const int32_t* __restrict__ idx,
                                                        const float* __restrict__ val, int64_t stride_k) {
  static_assert(kMergeTile <= 65536 && 2 * kMergeBitWords >= 2 * kMergeRepairCap, "key packing; the list fits");
  const int tid = threadIdx.x;
  uint32_t* once = s_multi;
  uint32_t* twice = s_multi + kMergeBitWords;
  uint32_t* thrice = s_multi + 2 * kMergeBitWords;
  uint32_t* flag = s_multi + 3 * kMergeBitWords;
  uint32_t* count = flag + 1;
  int pe[4];
  uint32_t off[4];
  float v[4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
    merge_entry((uint32_t)(r * 256 + tid), total, s_start, s_lo, td, sd, 0, np, idx, val, stride_k, pe[r], off[r],
                v[r]);
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    if (pe[r] >= 0 && off[r] < (uint32_t)td.n) {
      const uint32_t bit = 1u << (off[r] & 31u), wd = off[r] >> 5;
      if (atomicOr(&once[wd], bit) & bit)
        if (atomicOr(&twice[wd], bit) & bit) {
          atomicOr(&thrice[wd], bit);
          *flag = 1u;  // some element needs the repair
        }
      uint32_t* cell = reinterpret_cast<uint32_t*>(&s_acc[off[r]]);
      uint32_t seen = *cell;
      for (;;) {  // ends: a failed swap means another entry's swap succeeded
        const uint32_t want = __float_as_uint(__fadd_rn(__uint_as_float(seen), v[r]));
        const uint32_t got = atomicCAS(cell, seen, want);
        if (got == seen) break;
        seen = got;
      }
    }
  }
  __syncthreads();
  if (*flag == 0u) return true;  // uniform
  bool listed[4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
    listed[r] = pe[r] >= 0 && off[r] < (uint32_t)td.n && ((thrice[off[r] >> 5] >> (off[r] & 31u)) & 1u);
  __syncthreads();  // everybody has read `thrice` and the other bitmaps are dead: their space becomes the list
  uint32_t* lkey = s_multi;                                              // kMergeRepairCap words
  float* lval = reinterpret_cast<float*>(s_multi + kMergeRepairCap);     // kMergeRepairCap words
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    if (listed[r]) {
      const uint32_t at = atomicAdd(count, 1u);
      if (at < (uint32_t)kMergeRepairCap) {
        lkey[at] = off[r] | ((uint32_t)pe[r] << 16);
        lval[at] = v[r];
      }
    }
  }
  __syncthreads();
  const uint32_t n = *count;
  if (n > (uint32_t)kMergeRepairCap) return false;
  for (uint32_t i = tid; i < n; i += 256) {
    const uint32_t mine = lkey[i], o = mine & 0xFFFFu;
    bool first = true;
    for (uint32_t j = 0; j < n; ++j) first = first && !((lkey[j] & 0xFFFFu) == o && lkey[j] < mine);
    if (!first) continue;
    float sum = 0.0f;
    uint32_t last = 0u;  // keys of this element taken so far are below `last`
    for (;;) {
      uint32_t best = 0xFFFFFFFFu, bj = 0u;
      for (uint32_t j = 0; j < n; ++j) {
        const uint32_t kj = lkey[j];
        if ((kj & 0xFFFFu) == o && kj >= last && kj < best) { best = kj; bj = j; }
      }
      if (best == 0xFFFFFFFFu) break;
      sum = __fadd_rn(sum, lval[bj]);
      last = best + 0x10000u;  // the next worker's key at the earliest (worker numbers are below 256)
    }
    s_acc[o] = sum;
  }
  __syncthreads();
  return true;
}

template <typename T>
__device__ __forceinline__ uint32_t merge_accumulate(T* s_acc, uint32_t* s_start, int32_t* s_lo, uint32_t* s_wt,
                                                     uint32_t* s_multi, const TileDesc& td, const SegDesc& sd,
                                                     int slot, const int32_t* __restrict__ idx,
                                                     const float* __restrict__ val, int P, int64_t stride_k,
                                                     const int32_t* __restrict__ bounds) {
  const int tid = threadIdx.x;
  for (int i = tid; i < kMergeTile; i += 256) s_acc[i] = (T)0;
  if constexpr (sizeof(T) == 4) {
    if (P <= 256) {  // one batch of workers
      for (int i = tid; i < kMergeMultiWords; i += 256) s_multi[i] = 0u;
      const uint32_t total = merge_table(s_start, s_lo, s_wt, sd.k, slot, 0, P, P, bounds);
      if (total <= 1024u) {  // uniform over the workgroup
        if (merge_entries_unordered(s_acc, s_start, s_lo, s_multi, total, td, sd, P, idx, val, stride_k)) return total;
        for (int i = tid; i < kMergeTile; i += 256) s_acc[i] = (T)0;
        __syncthreads();
      }
      merge_entries_ordered<T>(s_acc, s_start, s_lo, total, td, sd, 0, P, idx, val, stride_k);
      return total;
    }
  }
  __syncthreads();
  uint32_t entries = 0;
  for (int p0 = 0; p0 < P; p0 += 256) {
    const int np = P - p0 < 256 ? P - p0 : 256;
    const uint32_t total = merge_table(s_start, s_lo, s_wt, sd.k, slot, p0, np, P, bounds);
    entries += total;
    merge_entries_ordered<T>(s_acc, s_start, s_lo, total, td, sd, p0, np, idx, val, stride_k);
  }
  return entries;
}

// k_merge<false>: the dense averaged update (Algorithm 1 lines 8-9): the whole tile is written
// once, divided by P.  k_merge<true>: the parameter step of Algorithm 1 line 9 applied in
// place, v -= update, touching only the elements whose sum is not zero (v - 0 == v bit for bit,
// and a sum that starts from +0.0f is never -0.0f).  No atomics, fixed summation order.
template <bool APPLY>
__global__ __launch_bounds__(256) void k_merge(const MTile* __restrict__ mtiles,
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
  __shared__ uint32_t s_multi[kMergeMultiWords];
  const MTile mt = mtiles[blockIdx.x];  // one read: the tile and what the kernel needs of its layer
  TileDesc td;
  td.start = mt.start; td.n = mt.n; td.seg = mt.seg; td.local0 = mt.local0; td.ctile = -1;
  SegDesc sd;
  sd.offset = 0; sd.out_offset = mt.out_offset; sd.d = 0; sd.k = mt.k;
  const int tid = threadIdx.x;
  const int slot = (int)blockIdx.x + td.seg;  // every earlier layer owns one extra (end) slot
  if (APPLY) s_claim[tid] = 0u;  // kMergeTile / 32 = 256 words; the accumulation's barriers order this
  const uint32_t entries =
      merge_accumulate<float>(s_acc, s_start, s_lo, s_wt, s_multi, td, sd, slot, idx, val, P, stride_k, bounds);
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
__global__ __launch_bounds__(256) void k_delta_tiles(const MTile* __restrict__ mtiles,
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
  const MTile mt = mtiles[blockIdx.x];
  TileDesc td;
  td.start = mt.start; td.n = mt.n; td.seg = mt.seg; td.local0 = mt.local0; td.ctile = -1;
  SegDesc sd;
  sd.offset = 0; sd.out_offset = mt.out_offset; sd.d = 0; sd.k = mt.k;
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const int slot = (int)blockIdx.x + td.seg;
  (void)merge_accumulate<double>(s_acc, s_start, s_lo, s_wt, nullptr, td, sd, slot, idx, val, P, stride_k, bounds);
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
      "k_prep", "k_small<4,1>", "k_small<4,8>", "k_stream", "k_group_h", "k_finish", "k_group_a",
      "k_group_p", "k_group_b",
      "k_hist", "k_count", "k_scan", "k_emit", "k_merge_bounds", "k_merge", "k_merge<apply>", "k_delta_tiles",
      "k_delta_finish", "sparsify_call"};
  return (id >= 0 && id < K_NUM) ? names[id] : nullptr;
}

__global__ void k_fill_u32(uint32_t* __restrict__ p, int64_t n, uint32_t value) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) p[i] = value;
}

hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t value, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, s, p, n, value);
  return hipGetLastError();
}

hipError_t launch_small(int cls, int nseg, const SegDesc* segs, const int32_t* list, const float* grad,
                        float* res, float lr, int32_t* out_idx, float* out_val, hipStream_t s, Prof* prof) {
  if (nseg <= 0) return hipSuccess;
  ProfScope ps(prof, K_SMALL0 + cls, s);
  if (cls == 0)
    hipLaunchKernelGGL((k_small<4, 1>), dim3(nseg), dim3(256), 0, s, segs, list, grad, res, lr, out_idx, out_val);
  else
    hipLaunchKernelGGL((k_small<4, 8>), dim3(nseg), dim3(256), 0, s, segs, list, grad, res, lr, out_idx, out_val);
  return hipGetLastError();
}

hipError_t launch_large_prep(const LargePlan& pl, const Scratch& sc, const SegDesc* segs, const float* grad,
                             const float* res, float lr, bool chain, hipStream_t s, Prof* prof) {
  if (pl.n_large <= 0) return hipSuccess;
  if (pl.has_dense) chain = true;
  uint32_t* counters = sc.ghist + (int64_t)pl.n_large * kHistStride;
  ProfScope ps(prof, K_PREP, s);
  hipLaunchKernelGGL(k_prep, dim3(pl.n_large), dim3(kPrepThreads), 0, s, segs, pl.lsegs, grad, res, lr, sc.lstate, sc.ghist,
                     counters, chain ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_large(const LargePlan& pl, const Scratch& sc, const SegDesc* segs, const float* grad,
                        float* res, float lr, int32_t* out_idx, float* out_val, bool chain, hipStream_t s,
                        Prof* prof, hipStream_t side, hipEvent_t side_ev) {
  if (pl.n_large <= 0) return hipSuccess;
  if (pl.has_dense) chain = true;
  uint32_t* counters = sc.ghist + (int64_t)pl.n_large * kHistStride;
  const int ch = chain ? 1 : 0;
  {
    const int nl = (pl.n_tiles + kStreamLaunchTiles - 1) / kStreamLaunchTiles;
    ProfScope ps(prof, K_STREAM, s, nl);
    for (int t0 = 0; t0 < pl.n_tiles; t0 += kStreamLaunchTiles) {
      const int nt = pl.n_tiles - t0 < kStreamLaunchTiles ? pl.n_tiles - t0 : kStreamLaunchTiles;
      hipLaunchKernelGGL((k_stream<kStreamWaves, kStreamV>), dim3(nt), dim3(kStreamWaves * 64), kStreamLdsPad, s,
                         pl.tiles + t0, grad, res, lr, sc.lstate, sc.chunk_cnt, sc.slots, pl.slot, sc.ghist);
    }
  }
  // Two launches share the layers (a list of layer indices each).  The small workgroups' layers
  // are finished by that launch alone, so it can run on the side stream beside the kernels of the
  // layers finished by groups; not when the multi-pass kernels follow, which read what it
  // appends to their work list.
  if (pl.n_finish_small > 0) {
    hipStream_t fs = s;
    if (side && !chain && pl.n_finish_small < pl.n_large) {
      if (hipEventRecord(side_ev, s) != hipSuccess || hipStreamWaitEvent(side, side_ev, 0) != hipSuccess)
        return hipErrorUnknown;
      fs = side;
    }
    ProfScope ps(prof, K_FINISH, fs);
    hipLaunchKernelGGL(k_finish<256>, dim3(pl.n_finish_small), dim3(256), 0, fs, pl.fin_small, segs, pl.lsegs, sc.lstate, sc.chunk_cnt,
                       sc.slots, pl.slot, sc.bh_part, sc.coarse_part, sc.part_info, res, out_idx, out_val, counters,
                       sc.items, ch, sc.fail_flag);
  }
  if (pl.n_hparts > 0) {
    ProfScope ps(prof, K_GROUP_H, s);
    hipLaunchKernelGGL(k_group_h, dim3(pl.n_hparts), dim3(1024), 0, s, pl.hparts, pl.lsegs, sc.lstate, sc.chunk_cnt,
                       sc.slots, pl.slot, sc.bh_part, sc.coarse_part, sc.part_info);
  }
  if (pl.n_finish_small < pl.n_large) {
    ProfScope ps(prof, K_FINISH, s);
    hipLaunchKernelGGL(k_finish<1024>, dim3(pl.n_large - pl.n_finish_small), dim3(1024), 0, s, pl.fin_other, segs, pl.lsegs, sc.lstate, sc.chunk_cnt,
                       sc.slots, pl.slot, sc.bh_part, sc.coarse_part, sc.part_info, res, out_idx, out_val, counters,
                       sc.items, ch, sc.fail_flag);
  }
  if (pl.n_groups > 0) {
    {
      ProfScope ps(prof, K_GROUP_A, s);
      hipLaunchKernelGGL(k_group_a, dim3(pl.n_groups), dim3(kGroupWaves * 64), 0, s, pl.groups, pl.lsegs, sc.lstate,
                         sc.chunk_cnt, sc.slots, pl.slot, sc.wgt, sc.band, sc.band_cnt);
    }
    {
      ProfScope ps(prof, K_GROUP_P, s);
      hipLaunchKernelGGL(k_group_p, dim3(pl.n_multi), dim3(1024), 0, s, pl.multi, segs, pl.lsegs, sc.lstate,
                         sc.chunk_cnt, sc.slots, pl.slot, sc.wgt, sc.band, sc.band_cnt, res, out_idx, out_val, counters,
                         sc.items, ch, sc.fail_flag);
    }
    ProfScope ps(prof, K_GROUP_B, s);
    hipLaunchKernelGGL(k_group_b, dim3(pl.n_groups), dim3(kGroupWaves * 64), 0, s, pl.groups, segs, pl.lsegs,
                       sc.lstate, sc.chunk_cnt, sc.slots, pl.slot, sc.wgt, res, out_idx, out_val);
  }
  if (chain) {
    const dim3 grid(kDenseGrid), b(256);
    // the digit chosen from each level's histogram is computed by the workgroups of the next launch
    for (int level = 0; level < 3; ++level) {
      ProfScope ps(prof, K_HIST, s);
      if (level == 0)
        hipLaunchKernelGGL((k_hist<0>), grid, b, 0, s, pl.tiles, sc.items, counters, pl.lsegs, segs, res, sc.dstate,
                           sc.ghist);
      else if (level == 1)
        hipLaunchKernelGGL((k_hist<1>), grid, b, 0, s, pl.tiles, sc.items, counters, pl.lsegs, segs, res, sc.dstate,
                           sc.ghist);
      else
        hipLaunchKernelGGL((k_hist<2>), grid, b, 0, s, pl.tiles, sc.items, counters, pl.lsegs, segs, res, sc.dstate,
                           sc.ghist);
    }
    {
      ProfScope ps(prof, K_COUNT, s);
      hipLaunchKernelGGL(k_count, grid, b, 0, s, pl.tiles, sc.items, counters, res, sc.dstate, sc.ghist, sc.tile_gt,
                         sc.tile_eq);
    }
    {
      ProfScope ps(prof, K_SCAN, s);
      hipLaunchKernelGGL(k_scan, dim3(pl.n_large), dim3(1024), 0, s, pl.lsegs, sc.lstate, sc.tile_gt, sc.tile_eq);
    }
    {
      ProfScope ps(prof, K_EMIT, s);
      hipLaunchKernelGGL(k_emit, grid, b, 0, s, pl.tiles, sc.items, counters, pl.lsegs, segs, res, sc.dstate,
                         sc.tile_gt, sc.tile_eq, out_idx, out_val);
    }
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
    hipLaunchKernelGGL((k_merge<false>), dim3(mp.n_mtiles), dim3(256), 0, s, mp.mtiles, idx, val, P, stride_k,
                       mp.nb, bounds, out);
  } else if (mode == MERGE_APPLY) {
    ProfScope ps(prof, K_MERGE_APPLY, s);
    hipLaunchKernelGGL((k_merge<true>), dim3(mp.n_mtiles), dim3(256), 0, s, mp.mtiles, idx, val, P, stride_k,
                       mp.nb, bounds, out);
  } else {
    {
      ProfScope ps(prof, K_DELTA_TILES, s);
      hipLaunchKernelGGL(k_delta_tiles, dim3(mp.n_mtiles), dim3(256), 0, s, mp.mtiles, res, res_stride, idx,
                         val, P, stride_k, mp.nb, bounds, partials);
    }
    ProfScope ps(prof, K_DELTA_FINISH, s);
    hipLaunchKernelGGL(k_delta_finish, dim3(mp.n_layers), dim3(256), 0, s, segs, mp.seg_mtile0, partials, out3);
  }
  return hipGetLastError();
}

}  // namespace lags
