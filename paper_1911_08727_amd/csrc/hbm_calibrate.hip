// libhbmcal.so: plain streaming kernels that measure what HBM bandwidth a kernel of the
// streaming pass's shape can reach on this GPU: the practical ceiling beside the 8 TB/s of
// the data sheet.  Measurement aid only: nothing of the method is in here and liblags.so
// does not use it.
//
// Shape of every kernel = shape of the sparsifier's streaming pass: workgroups of 256 threads,
// one tile of 4096 floats per workgroup (a wave walks 1024 consecutive floats in 4 rounds of
// 64 lanes x 16 bytes), non-temporal 16-byte accesses, back-to-back launches of at most 65536
// tiles, an optional amount of unused dynamic LDS per workgroup that caps the workgroups per CU.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kTile = 4096;
constexpr int kLaunchTiles = 65536;

enum { CAL_COPY = 0, CAL_READ = 1, CAL_TRIAD = 2, CAL_WRITE = 3 };

// KIND 0: b = a (8 bytes per element); 1: read a only (4); 2: b = b + lr * a in two roundings, the
// accumulate of Algorithm 1 line 6 (12); 3: write b only (4).
template <int KIND>
__global__ __launch_bounds__(256) void k_cal(const float* __restrict__ a, float* __restrict__ b, float lr,
                                             int64_t tile0, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t base = (tile0 + blockIdx.x) * kTile + w * 1024;
  f32x4 av[4], bv[4];
  if (KIND != CAL_WRITE) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = j * 256 + lane * 4;
      av[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a + base + e));
      if (KIND == CAL_TRIAD) bv[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(b + base + e));
    }
  }
  if (KIND == CAL_READ) {
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) s += (av[j].x + av[j].y) + (av[j].z + av[j].w);
    if (s == 12345.678f) sink[0] = s;  // keeps the loads alive; practically never true
    return;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = j * 256 + lane * 4;
    f32x4 o;
    if (KIND == CAL_COPY) {
      o = av[j];
    } else if (KIND == CAL_TRIAD) {
      float t0 = __fmul_rn(lr, av[j].x), t1 = __fmul_rn(lr, av[j].y), t2 = __fmul_rn(lr, av[j].z),
            t3 = __fmul_rn(lr, av[j].w);
      asm volatile("" : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3));
      o.x = __fadd_rn(bv[j].x, t0);
      o.y = __fadd_rn(bv[j].y, t1);
      o.z = __fadd_rn(bv[j].z, t2);
      o.w = __fadd_rn(bv[j].w, t3);
    } else {
      o.x = lr; o.y = lr; o.z = lr; o.w = lr;
    }
    __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(b + base + e));
  }
}

template <int KIND>
hipError_t enqueue(const float* a, float* b, int64_t n_tiles, int lds_pad, hipStream_t s, float* sink) {
  for (int64_t t0 = 0; t0 < n_tiles; t0 += kLaunchTiles) {
    const int64_t nt = n_tiles - t0 < kLaunchTiles ? n_tiles - t0 : kLaunchTiles;
    hipLaunchKernelGGL((k_cal<KIND>), dim3((unsigned)nt), dim3(256), lds_pad, s, a, b, 0.1f, t0, sink);
  }
  return hipGetLastError();
}

}  // namespace

extern "C" {

// Runs kernel `kind` (0 copy b = a, 1 read a, 2 triad b += 0.1 a, 3 write b) `reps` times over
// n_elems floats (a multiple of 4096; a and b device arrays of at least that many floats, 16-byte
// aligned, not overlapping; sink a device float) on `hip_stream`, after one untimed run, and
// returns the average milliseconds per run in *ms (HIP events on that stream; the call waits for
// them).  lds_pad: bytes of unused dynamic LDS per workgroup (0..65536).  Returns 0, or -1 on a
// bad argument, -3 on a HIP error.
int hbmcal_time(int kind, const float* a, float* b, float* sink, int64_t n_elems, int reps, int lds_pad,
                void* hip_stream, float* ms) {
  if (!a || !b || !sink || !ms || kind < 0 || kind > 3 || n_elems < kTile || n_elems % kTile != 0 || reps < 1 ||
      lds_pad < 0 || lds_pad > 65536)
    return -1;
  if (((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15u) != 0) return -1;
  hipStream_t s = (hipStream_t)hip_stream;
  const int64_t n_tiles = n_elems / kTile;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
    if (e0) (void)hipEventDestroy(e0);
    return -3;
  }
  hipError_t err = hipSuccess;
  for (int r = -1; r < reps && err == hipSuccess; ++r) {
    if (r == 0) err = hipEventRecord(e0, s);
    if (err != hipSuccess) break;
    if (kind == CAL_COPY) err = enqueue<CAL_COPY>(a, b, n_tiles, lds_pad, s, sink);
    else if (kind == CAL_READ) err = enqueue<CAL_READ>(a, b, n_tiles, lds_pad, s, sink);
    else if (kind == CAL_TRIAD) err = enqueue<CAL_TRIAD>(a, b, n_tiles, lds_pad, s, sink);
    else err = enqueue<CAL_WRITE>(a, b, n_tiles, lds_pad, s, sink);
  }
  float total = 0.f;
  if (err == hipSuccess) err = hipEventRecord(e1, s);
  if (err == hipSuccess) err = hipEventSynchronize(e1);
  if (err == hipSuccess) err = hipEventElapsedTime(&total, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (err != hipSuccess) return -3;
  *ms = total / (float)reps;
  return 0;
}

}  // extern "C"
