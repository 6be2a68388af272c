// Internal declarations shared by the host API (lags_api.hip) and the kernels
// (lags_kernels.hip).  Not part of the public interface.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

namespace lags {

// Geometry of the multi-block ("large") path: one workgroup of 4 waves per tile,
// each wave owns a contiguous quarter of the tile and walks it in rounds of
// 64 lanes x 4 consecutive elements.
constexpr int kTileWaves = 4;
constexpr int kTileV = 8;                               // rounds per wave
constexpr int kWaveChunk = kTileV * 256;                // 2048 elements per wave
constexpr int kTile = kTileWaves * kWaveChunk;          // 8192 elements per tile
constexpr int kBins0 = 2048;                            // key bits 30..20
constexpr int kBins12 = 1024;                           // key bits 19..10, 9..0
constexpr int kHistStride = 2048;

// Size classes of the one-workgroup-per-layer ("small") path: NW waves x V rounds.
constexpr int kSmall0 = 4 * 1 * 256;     // <= 1024  : 4 waves, 1 round
constexpr int kSmall1 = 4 * 8 * 256;     // <= 8192  : 4 waves, 8 rounds
constexpr int kSmall2 = 16 * 10 * 256;   // <= 40960 : 16 waves, 10 rounds

constexpr int kMergeTile = 8192;
constexpr int kMaxWorkers = 1024;

struct SegDesc {        // one layer
  int64_t offset;       // element offset in the flat arrays
  int64_t out_offset;   // position of the layer's pairs in out_idx/out_val
  int32_t d;
  int32_t k;
};

struct TileDesc {       // one tile of a layer
  int64_t start;        // absolute element offset of the tile's first element
  int32_t n;            // valid elements in the tile (<= tile size)
  int32_t seg;          // large path: index among the large layers; merge: layer index
  int32_t local0;       // layer-local index of the tile's first element
  int32_t pad;
};

struct LargeSeg {
  int32_t seg;          // layer index
  int32_t tile_begin;   // first tile of the layer in the tile list
  int32_t tile_end;
  int32_t pad;
};

struct SegState {       // radix-select state of one large layer
  uint32_t prefix;      // key bits decided so far
  uint32_t k_rem;       // entries still to take among keys matching the prefix
};

// Kernel ids for the optional event timing.
enum KernelId {
  K_ZERO = 0, K_SMALL0, K_SMALL1, K_SMALL2, K_ACCUM_HIST, K_CHOOSE, K_HIST, K_COUNT, K_SCAN, K_EMIT,
  K_MERGE, K_NUM
};
const char* kernel_name(int id);

struct Prof {
  bool on = false;
  struct Rec { int id; hipEvent_t a, b; };
  std::vector<Rec> recs;
};

// Brackets one kernel launch with events when profiling is on.
struct ProfScope {
  Prof* p; hipStream_t s; hipEvent_t a = nullptr, b = nullptr; int id;
  ProfScope(Prof* prof, int kid, hipStream_t st) : p(prof && prof->on ? prof : nullptr), s(st), id(kid) {
    if (p && hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess) (void)hipEventRecord(a, s);
    else p = nullptr;
  }
  ~ProfScope() {
    if (p) { (void)hipEventRecord(b, s); p->recs.push_back(Prof::Rec{id, a, b}); }
  }
};

// Launch wrappers (lags_kernels.hip).  All enqueue on `s` and return the launch status.
hipError_t launch_zero_u32(uint32_t* p, int64_t n, hipStream_t s, Prof* prof);
hipError_t launch_small(int cls, int nseg, const SegDesc* segs, const int32_t* list, const float* grad,
                        float* res, float lr, int32_t* out_idx, float* out_val, hipStream_t s, Prof* prof);
hipError_t launch_large(int n_large, int n_tiles, const SegDesc* segs, const LargeSeg* lsegs,
                        const TileDesc* tiles, const float* grad, float* res, float lr,
                        int32_t* out_idx, float* out_val, uint32_t* ghist, SegState* state,
                        uint32_t* tile_gt, uint32_t* tile_eq, hipStream_t s, Prof* prof);
hipError_t launch_merge(int n_tiles, const TileDesc* mtiles, const SegDesc* segs, const int32_t* idx,
                        const float* val, int P, int64_t stride_k, float* update, hipStream_t s, Prof* prof);

}  // namespace lags
