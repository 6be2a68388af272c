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
// Anything larger goes through the sampled pipeline: a single workgroup that held a layer of
// tens of thousands of elements in registers ran for 40 us and took a whole CU's registers from
// the streaming pass meanwhile.
constexpr int kSmallClasses = 2;

// Threshold guess from a sample (large layers): 256 pieces of 64 consecutive elements.
// The sample only has to rank the top k roughly: a smaller sample admits more candidates
// (the threshold sits five standard deviations of the sample count below the top k), which
// costs 8 bytes each and little else.
constexpr int kSamplePiece = 64;
constexpr int kSamplePieces = 256;
constexpr int kSampleMax = kSamplePiece * kSamplePieces;   // 16384 sampled elements
// Layers of up to kSampleSmallElems elements are guessed from a quarter of that.  The sample is
// read from scattered 256-byte pieces before the streaming pass can start; a shorter one admits
// more candidates (its threshold is less sharp), and below about two million elements the bytes
// saved on the sample outweigh the bytes of the extra candidates.
constexpr int kSamplePiecesSmall = 64;
constexpr int64_t kSampleSmallElems = 1 << 20;
constexpr int kSlotMin = 128;            // candidate slots per tile of a sampled layer: the table uses the
constexpr int kSlotMax = 2048;           // smallest power of two >= 8x the expected count of any layer
constexpr int kDenseGrid = 1024;         // workgroups of the multi-pass kernels (grid-stride)
// Finish of a sampled layer.  The candidates are counted in kFineBins buckets of 2^shift key
// steps above the threshold tau; the buckets cover the part of the key range where the k-th
// largest key is expected, candidates above it are counted in one number.  The bucket that
// holds the k-th largest key is then resolved exactly among its own entries ("band"), which
// must number at most kBandCap.
constexpr int kFineBins = 4096;
constexpr int kBandCap = 4096;
constexpr int kBandCapSmall = 1024;        // ... of the layers that k_finish takes with workgroups of 256 threads
constexpr int kWaveTiles = 8;            // a wave flattens the slots of 8 consecutive tiles ("wave chunk")
constexpr int kGroupWaves = 8;           // a workgroup of the multi-workgroup finish: 8 wave chunks
constexpr int kGroupTiles = kWaveTiles * kGroupWaves;
constexpr int kGroupBand = 64;           // band entries one group may contribute
constexpr int kCountTiles = 256;         // tiles per workgroup of the partial bucket counts
constexpr int kCoarseBins = 64;          // those counts are also summed over runs of 64 buckets
constexpr int kFusedTiles = 512;         // sampled layers of up to this many tiles are finished by one workgroup
// ... unless the table also holds a sampled layer above kFusedTiles: the launches of the finish
// by groups are then paid anyway, and a single workgroup walking hundreds of tiles would be the
// longest thing in k_finish.  Such tables keep only layers of up to this many tiles in one workgroup.
constexpr int kFusedTilesShared = 128;
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
constexpr int kBoundChunk = 2048;        // index-list entries per workgroup of k_merge_bounds


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

struct TileDesc {       // one tile of a layer (dense tiles, merge tiles)
  int64_t start;        // absolute element offset
  int32_t n;            // elements in the tile (<= tile size)
  int32_t seg;          // large path: index among the large layers; merge: layer index
  int32_t local0;       // layer-local index of the first element
  int32_t ctile;        // dense tiles of sampled layers: index among those tiles ("chunk"); else -1
};

struct MTile {          // one tile of the dense update (merge-type kernels), with what they need of its layer
  int64_t start;        // absolute element offset
  int64_t out_offset;   // position of the layer's pairs in a worker's idx/val
  int32_t n;            // elements in the tile
  int32_t seg;          // layer index
  int32_t local0;       // layer-local index of the first element
  int32_t k;            // pairs per worker of the layer
};

struct LargeSeg {       // static plan of one large layer
  int32_t seg;          // layer index
  int32_t tile_begin;   // dense tiles [tile_begin, tile_end)
  int32_t tile_end;
  int32_t sampled;      // 1: threshold guess from a sample, candidates collected in slots
  int32_t chunk_begin;  // sampled layers: their tiles' ctile numbers [chunk_begin, chunk_end), else 0,0
  int32_t chunk_end;
  int32_t fused;        // sampled layers: 1 = finished by one workgroup, 0 = by groups of tiles
  int32_t wchunk_begin; // sampled layers: first of the layer's wave chunks in the per-wave-chunk array
  int32_t group_begin;  // multi-workgroup finish: the layer's groups [group_begin, group_end)
  int32_t group_end;
  int32_t group_h_begin;  // ... and its parts of the bucket counts [group_h_begin, group_h_end)
  int32_t group_h_end;
  int32_t sample_rank;  // rank (1-based, from the top) of the sample key used as threshold tau
  int32_t sample_rank_hi;  // rank of the sample key that estimates the layer's k-th largest key
  int32_t sample_pieces;
  int32_t sample_stride;
};

// Sampled layers of at most this many tiles that one workgroup finishes are finished by one of
// 256 threads instead of 1024 (four wave chunks per wave at most): a CU holds six of those
// side by side, against two of the large ones, and a table of many layers is done sooner.
constexpr int kFinishSmallTiles = 128;
__host__ __device__ inline bool finish_small(const LargeSeg& ls) {
  return ls.sampled && ls.fused && ls.chunk_end - ls.chunk_begin <= kFinishSmallTiles;
}

struct GroupDesc {      // one workgroup of the multi-workgroup finish (a group, or a part of the bucket counts)
  int32_t lseg;         // large-layer index
  int32_t first;        // index of the group (part) inside its layer
};

enum : uint32_t { MODE_DENSE = 0, MODE_SPARSE = 1 };

struct LState {         // per call, per large layer
  uint32_t tau;         // candidates are the entries with key >= tau
  uint32_t t_zero;      // candidates with key >= t_zero had their residual zeroed by the streaming pass
  uint32_t tau_top;     // candidates with key >= tau_top are counted in one number, the others per bucket
  uint32_t shift;       // bucket of a candidate below tau_top: (key - tau) >> shift
  uint32_t mode;        // MODE_SPARSE: the guess held, the slots contain the top k
  uint32_t bstar;       // the bucket that holds the k-th largest key
  uint32_t k_rem;       // how many of that bucket's entries belong to the top k
  uint32_t n_band;      // entries in that bucket
  uint32_t band_over;   // a group collected more band entries than it can hold
  uint32_t route;       // for lags_last_routes: 1 accepted, 2 rejected, 3 not sampled
  uint32_t T, I;        // multi-workgroup finish: kept = key > T, or key == T and index <= I

};

struct DState {         // per call, per large layer on the multi-pass route: the radix select's progress
  uint32_t p0, k0;      // after digit 0: key bits decided, entries still to take below them
  uint32_t p1, k1;      // ... after digit 1
  uint32_t prefix;      // ... after digit 2: the k-th largest key T
  uint32_t k_rem;       //     and how many entries equal to T belong to the top k
  uint32_t pad[2];
};

struct LargePlan {      // everything launch_large needs (device pointers + counts)
  int n_large = 0, n_tiles = 0, n_sampled = 0, n_chunks = 0, n_wchunks = 0, n_groups = 0, n_multi = 0, n_hparts = 0;
  int n_finish_small = 0;               // large layers that k_finish takes with workgroups of 256 threads
  int slot = kSlotMin;                  // candidate slots per sampled tile
  bool has_dense = false;               // some large layer is not sampled: the multi-pass kernels always run
  const LargeSeg* lsegs = nullptr;
  const TileDesc* tiles = nullptr;      // dense tiles
  const GroupDesc* groups = nullptr;    // groups of the layers with fused == 0
  const GroupDesc* hparts = nullptr;    // parts of their bucket counts
  const int32_t* multi = nullptr;       // large-layer indices of those layers
  const int32_t* fin_small = nullptr;   // large-layer indices that k_finish<256> takes (n_finish_small)
  const int32_t* fin_other = nullptr;   // ... and the others (n_large - n_finish_small), for k_finish<1024>
};

struct Scratch {        // context-owned device memory, contents meaningless between calls
  uint32_t* bh_part = nullptr;    // n_hparts * kFineBins: partial bucket counts
  uint32_t* coarse_part = nullptr;  // n_hparts * kCoarseBins: their sums over runs of 64 buckets
  uint4* part_info = nullptr;     // n_hparts: candidates, candidates at or above tau_top, overflow flag
  LState* lstate = nullptr;       // n_large
  uint32_t* chunk_cnt = nullptr;  // n_chunks: candidates of the tile
  uint2* slots = nullptr;         // n_chunks * slot
  uint32_t* wgt = nullptr;        // n_wchunks: entries above the decisive bucket per wave chunk, then output positions
  uint2* band = nullptr;          // n_groups * kGroupBand
  uint32_t* band_cnt = nullptr;   // n_groups
  // multi-pass route (layers that are not sampled, rejected guesses)
  uint32_t* ghist = nullptr;      // n_large * kHistStride, then 16 counters ([0] = number of work items)
  DState* dstate = nullptr;       // n_large
  uint32_t* tile_gt = nullptr;    // n_tiles
  uint32_t* tile_eq = nullptr;
  int32_t* items = nullptr;       // n_tiles: dense tiles to process
  uint32_t* fail_flag = nullptr;  // device address of the context's pinned host word
};

// Kernel ids for the optional event timing.
enum KernelId {
  K_PREP = 0, K_SMALL0, K_SMALL1, K_STREAM, K_GROUP_H, K_FINISH, K_GROUP_A, K_GROUP_P, K_GROUP_B,
  K_HIST, K_COUNT, K_SCAN, K_EMIT,
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

// Planning shared by the table builder and the entry point that allocates nothing (lags_api.hip).
// plan_sample: the sample plan of a large layer of d elements keeping k (fills the sample_*
// fields of *ls); false if the layer is not worth sampling.  *per_tile = expected candidates
// per tile.  plan_slots: candidate slots per tile for the largest such expectation of a table.
bool plan_sample(int64_t d, int64_t k, LargeSeg* ls, double* per_tile);
int plan_slots(double max_per_tile);

// Launch wrappers (lags_kernels.hip).  All enqueue on `s` and return the launch status.
hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t value, hipStream_t s);
hipError_t launch_small(int cls, int nseg, const SegDesc* segs, const int32_t* list, const float* grad,
                        float* res, float lr, int32_t* out_idx, float* out_val, hipStream_t s, Prof* prof);
// The large layers' pipeline in two parts, same arguments to both: the threshold guesses
// (k_prep), then everything that follows them.  chain: also enqueue the multi-pass kernels
// (rejected guesses then use them instead of the one-workgroup rescue); always true for plans
// with has_dense.  side (may be null): a second stream on which launch_large may enqueue work
// that depends only on the streaming pass, after an event `side_ev` that it records on `s`; the
// caller joins `side` to `s` afterwards.
hipError_t launch_large_prep(const LargePlan& pl, const Scratch& sc, const SegDesc* segs, const float* grad,
                             const float* res, float lr, bool chain, hipStream_t s, Prof* prof);
hipError_t launch_large(const LargePlan& pl, const Scratch& sc, const SegDesc* segs, const float* grad,
                        float* res, float lr, int32_t* out_idx, float* out_val, bool chain, hipStream_t s,
                        Prof* prof, hipStream_t side = nullptr, hipEvent_t side_ev = nullptr);
enum { MERGE_UPDATE = 0, MERGE_APPLY = 1, MERGE_DELTA = 2 };

struct MergePlan {      // device pointers + counts of the merge-type launches
  int n_layers = 0, n_mtiles = 0, n_bchunks = 0, nb = 0;
  const MTile* mtiles = nullptr;
  const BChunk* bchunks = nullptr;
  const int32_t* seg_mtile0 = nullptr;  // n_layers + 1: first merge tile of every layer
};

// mode MERGE_UPDATE: out = dense update; MERGE_APPLY: out = parameters, updated in place;
// MERGE_DELTA: res/res_stride/partials/out3 are used instead of out.
hipError_t launch_merge(int mode, const MergePlan& mp, int32_t* bounds, const SegDesc* segs, const int32_t* idx,
                        const float* val, int P, int64_t stride_k, float* out, const float* res,
                        int64_t res_stride, double* partials, double* out3, hipStream_t s, Prof* prof);

}  // namespace lags
