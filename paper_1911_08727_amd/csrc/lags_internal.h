// Internal declarations shared by the host API (lags_api.hip) and the kernels
// (lags_kernels.hip).  Not part of the public interface.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

namespace lags {

// Geometry of the multi-block ("large") path: one workgroup of 4 waves per tile,
// each wave owns a contiguous quarter of the tile and walks it in rounds of 64 lanes x 4
// consecutive elements.  A tile of a sampled layer is also the unit ("chunk") that owns
// `slot` candidate slots (a power of two between kSlotMin and kSlotMax chosen per table).
constexpr int kTileWaves = 4;
constexpr int kTileV = 4;                               // rounds per wave
constexpr int kWaveChunk = kTileV * 256;                // 1024 elements per wave
constexpr int kTile = kTileWaves * kWaveChunk;          // 4096 elements per tile
constexpr int kBins0 = 2048;                            // key bits 30..20
constexpr int kBins12 = 1024;                           // key bits 19..10, 9..0
constexpr int kHistLevel1 = kBins0;                     // a layer's three histograms sit side by side:
constexpr int kHistLevel2 = kBins0 + kBins12;           // level 0 at [0, 2048), level 1 at [2048, 3072),
constexpr int kHistStride = kBins0 + 2 * kBins12;       // level 2 at [3072, 4096)

// Size classes of the one-workgroup-per-layer ("small") path: NW waves x V rounds.
constexpr int kSmall0 = 4 * 1 * 256;     // <= 1024  : 4 waves, 1 round
constexpr int kSmall1 = 4 * 8 * 256;     // <= 8192  : 4 waves, 8 rounds
constexpr int kSmall2 = 16 * 10 * 256;   // <= 40960 : 16 waves, 10 rounds

// Threshold guess from a sample (large layers): 256 pieces of 64 consecutive elements.
// The sample only has to rank the top k roughly: a smaller sample admits more candidates
// (the threshold sits four standard deviations of the sample count below the top k), which
// costs 8 bytes each and nothing else.
constexpr int kSamplePiece = 64;
constexpr int kSamplePieces = 256;
constexpr int kSampleMax = kSamplePiece * kSamplePieces;   // 16384 sampled elements
// Layers that keep many entries (k >= kBigSampleK) of many elements take four times the sample:
// the threshold is then tighter (about 1.6 k candidates instead of 2.5 k at rho = 0.001), which
// saves more candidate traffic than the larger sample costs.
constexpr int kSamplePieceBig = 256;                       // 256 pieces x 256 = 65536 sampled elements
constexpr int kBigSampleK = 8192;
constexpr int64_t kBigSampleD = 1 << 20;
constexpr int kSlotMin = 128;            // candidate slots per tile of a sampled layer: the table uses the
constexpr int kSlotMax = 2048;           // smallest power of two >= 8x the expected count of any layer
constexpr int kDenseGrid = 1024;         // workgroups of the fallback kernels (grid-stride)
// The streaming pass is HBM-bound and runs best when each CU holds only three of its
// workgroups (12 waves, about 96 KB of loads in flight per CU): measured on MI355X, 26.6 GB in
// 4.05 ms, against 4.36 ms at the eight workgroups that registers and static LDS would allow
// (more bytes in flight only widen the window of DRAM rows that are open at once) and 4.6 ms
// at two.  The launch therefore asks for this much unused dynamic LDS per workgroup, which
// caps the workgroups per CU at three (160 KB of LDS per CU).
constexpr int kStreamLdsPad = 40960;
// It is enqueued as back-to-back launches of at most this many tiles: with the occupancy cap,
// launches of 65536 tiles measured 3 % faster than one launch of 540000 tiles and 2 % faster than
// launches of 16384 (a launch boundary lets the 8 XCDs, which drift apart inside a launch, start
// again from neighbouring addresses).
constexpr int kStreamLaunchTiles = 65536;
// Shape of the streaming workgroup: 4 waves x 4 rounds (8 x 2 and 2 x 8 measured 2-4 % slower at
// their best occupancy, 16 x 1 10 % slower).
constexpr int kStreamWaves = 4;
constexpr int kStreamV = 4;

constexpr int kMergeTile = 8192;
constexpr int kMaxWorkers = 1024;
constexpr int kBoundChunk = 16384;       // index-list entries per workgroup of k_merge_bounds

struct BChunk {         // a run of one layer's index list, for k_merge_bounds
  int32_t seg;          // layer
  int32_t j0;           // first list position of the run
  int32_t slot0;        // the layer's first slot in a worker's bounds row
  int32_t ntiles;       // merge tiles of the layer
};

struct SegDesc {        // one layer
  int64_t offset;       // element offset in the flat arrays
  int64_t out_offset;   // position of the layer's pairs in out_idx/out_val
  int32_t d;
  int32_t k;
};

struct TileDesc {       // one tile of a layer (dense tiles, candidate tiles, merge tiles)
  int64_t start;        // dense/merge: absolute element offset; candidate tile: offset in the candidate array
  int32_t n;            // elements in the tile (<= tile size); candidate tiles: capacity
  int32_t seg;          // large path: index among the large layers; merge: layer index
  int32_t local0;       // layer-local index (candidate tiles: list position) of the first element
  int32_t ctile;        // dense tiles of sampled layers: index among those tiles ("chunk"); else -1
};

enum : int32_t { CAND_NONE = 0, CAND_SMALL0 = 1, CAND_SMALL1 = 2, CAND_SMALL2 = 3, CAND_LARGE = 4 };

struct LargeSeg {       // static plan of one large layer
  int64_t cand_base;    // start of the layer's candidate list in the candidate array
  int32_t seg;          // layer index
  int32_t tile_begin;   // dense tiles [tile_begin, tile_end)
  int32_t tile_end;
  int32_t chunk_begin;  // sampled layers: their tiles' ctile numbers [chunk_begin, chunk_end), else 0,0
  int32_t chunk_end;
  int32_t cand_class;   // CAND_NONE: not sampled
  int32_t cap;          // capacity of the candidate list
  int32_t ctile_begin;  // candidate tiles (CAND_LARGE) [ctile_begin, ctile_end)
  int32_t ctile_end;
  int32_t sample_rank;  // rank (1-based, from the top) of the sample key used as threshold tau
  int32_t sample_rank_hi;  // rank of the sample key used as tau_hi (0: none): about k's share of the sample
  int32_t sample_pieces;
  int32_t sample_stride;
  int32_t sample_big;   // 1: pieces of kSamplePieceBig elements (the large sample), 0: of kSamplePiece
};

enum : uint32_t { MODE_DENSE = 0, MODE_SPARSE = 1 };

struct LState {         // per call, per large layer
  uint32_t tau;         // candidates are the entries with key >= tau
  uint32_t tau_hi;      // candidates with key >= tau_hi had their residual zeroed by the streaming pass
  uint32_t ncand;       // number of candidates found
  uint32_t mode;        // MODE_SPARSE: the candidate list holds the top k; MODE_DENSE: fall back
  uint32_t p0, k0;      // radix select after digit 0: key bits decided, entries still to take below them
  uint32_t p1, k1;      // ... after digit 1
  uint32_t prefix;      // ... after digit 2: the k-th largest key T
  uint32_t k_rem;       //     and how many entries equal to T belong to the top k
  uint32_t pad[2];
};

struct LargePlan {      // everything launch_large needs (device pointers + counts)
  int n_large = 0, n_tiles = 0, n_sampled = 0, n_chunks = 0, n_ctiles = 0;
  int slot = kSlotMin;                  // candidate slots per sampled tile
  bool big_sample = false;              // some layer uses the large sample
  int n_cand_small[3] = {0, 0, 0};
  const LargeSeg* lsegs = nullptr;
  const TileDesc* tiles = nullptr;      // dense tiles
  const TileDesc* ctiles = nullptr;     // candidate tiles of CAND_LARGE layers
  const int32_t* sampled = nullptr;     // large-layer indices that are sampled
  const int32_t* cand_small[3] = {nullptr, nullptr, nullptr};  // large-layer indices per class
  const int32_t* chunk_lseg = nullptr;  // chunk (sampled tile) -> large-layer index
};

struct Scratch {        // context-owned device memory, contents meaningless between calls
  uint32_t* ghist = nullptr;      // n_large * kHistStride, then 16 counters ([0] = number of dense
                                  // work items); zeroed each call
  LState* lstate = nullptr;       // n_large
  uint32_t* tile_gt = nullptr;    // n_tiles + n_ctiles
  uint32_t* tile_eq = nullptr;
  int32_t* items = nullptr;       // n_tiles: dense tiles to process in fallback mode
  uint32_t* chunk_cnt = nullptr;  // n_chunks
  uint32_t* chunk_off = nullptr;  // n_chunks
  uint2* slots = nullptr;         // n_chunks * slot
  uint2* cand = nullptr;          // sum of cap over sampled layers
};

// Kernel ids for the optional event timing.
enum KernelId {
  K_ZERO = 0, K_SMALL0, K_SMALL1, K_SMALL2, K_SAMPLE, K_STREAM, K_CSCAN, K_CGATHER,
  K_CSMALL0, K_CSMALL1, K_CSMALL2, K_HIST, K_COUNT, K_SCAN, K_EMIT,
  K_MERGE_BOUNDS, K_MERGE, K_MERGE_APPLY, K_DELTA_TILES, K_DELTA_FINISH,
  K_SPARSIFY_CALL,      // not a kernel: the whole sparsify call on the caller's stream, fork to join
  K_NUM
};
const char* kernel_name(int id);

struct Prof {
  bool on = false;
  int only = -1;        // >= 0: record this kernel id only
  struct Rec { int id; hipEvent_t a, b; int launches; };
  std::vector<Rec> recs;
};

// Brackets one kernel launch (or one back-to-back group of launches of the same kernel) with
// events when profiling is on.
struct ProfScope {
  Prof* p; hipStream_t s; hipEvent_t a = nullptr, b = nullptr; int id; int launches;
  ProfScope(Prof* prof, int kid, hipStream_t st, int nlaunch = 1)
      : p(prof && prof->on && (prof->only < 0 || prof->only == kid) ? prof : nullptr), s(st), id(kid),
        launches(nlaunch) {
    if (p && hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess) (void)hipEventRecord(a, s);
    else p = nullptr;
  }
  ~ProfScope() {
    if (p) { (void)hipEventRecord(b, s); p->recs.push_back(Prof::Rec{id, a, b, launches}); }
  }
};

// Launch wrappers (lags_kernels.hip).  All enqueue on `s` and return the launch status.
hipError_t launch_zero_u32(uint32_t* p, int64_t n, hipStream_t s, Prof* prof);
hipError_t launch_small(int cls, int nseg, const SegDesc* segs, const int32_t* list, const float* grad,
                        float* res, float lr, int32_t* out_idx, float* out_val, hipStream_t s, Prof* prof);
hipError_t launch_large(const LargePlan& pl, const Scratch& sc, const SegDesc* segs, const float* grad,
                        float* res, float lr, int32_t* out_idx, float* out_val, hipStream_t s, Prof* prof);
enum { MERGE_UPDATE = 0, MERGE_APPLY = 1, MERGE_DELTA = 2 };

struct MergePlan {      // device pointers + counts of the merge-type launches
  int n_layers = 0, n_mtiles = 0, n_bchunks = 0, nb = 0;
  const TileDesc* mtiles = nullptr;
  const BChunk* bchunks = nullptr;
  const int32_t* seg_mtile0 = nullptr;  // n_layers + 1: first merge tile of every layer
};

// mode MERGE_UPDATE: out = dense update; MERGE_APPLY: out = parameters, updated in place;
// MERGE_DELTA: res/res_stride/partials/out3 are used instead of out.
hipError_t launch_merge(int mode, const MergePlan& mp, int32_t* bounds, const SegDesc* segs, const int32_t* idx,
                        const float* val, int P, int64_t stride_k, float* out, const float* res,
                        int64_t res_stride, double* partials, double* out3, hipStream_t s, Prof* prof);

}  // namespace lags
