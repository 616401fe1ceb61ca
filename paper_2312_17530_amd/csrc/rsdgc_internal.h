// Internal definitions shared by the host-side plan and the HIP kernels.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/rsdgc.h"

namespace rsdgc {

// ---- geometry constants (device and host agree on these) -----------------
constexpr int kTileRows = 16;        // NSI tile: output rows per workgroup
constexpr int kTileCols = 256;       // NSI tile: output columns per workgroup
constexpr int kChunk = 8192;         // elements per workgroup in the 1-D passes
constexpr int kHistBins = 4096;      // widest radix digit (12 bits)
constexpr int kLayerAlign = 64;      // arena alignment of a layer, in elements
constexpr int kSlotCapMax = 512;     // candidate centres one tile of a layer on the candidate path can record
constexpr int kSlotGroup = 16;       // tile slots per work item of the candidate passes (one per wave)
constexpr int kFineShift = 13;       // candidate path: the first ranking digit counts score bits in steps of 2^13
constexpr int kFineBins = 1024;      // ... relative to the candidate bound: 1024 bins = one binade above it
constexpr int kLevel1Bits = 11;      // second ranking digit (both paths)
constexpr int kLevel1Bins = 1 << kLevel1Bits;
constexpr int kCoarseShift = 19;     // full-map path: the first digit is the top 12 bits of the 31-bit score
constexpr int kListMin = 8192;       // smallest threshold-bucket list of a layer (entries)
constexpr int kListDiv = 32;         // ... or 1/32 of the layer, whichever is larger
constexpr int kCountChunks = 16;     // chunks per workgroup of the count pass
constexpr int kChunkGroup = 64;      // chunks per group in the two-level chunk prefix
constexpr int kListShards = 16;      // a layer's threshold-bucket list is filled through this many counters
constexpr int kGroupCntStride = 32;   // words between two chunk-group counters where many workgroups add to one: a cache line each
constexpr uint32_t kInlineCountChunks = 4096;   // plans up to this many chunks (33 M elements) count their kept elements where the bits are set
constexpr int kListCntStride = 32;   // uint32 between two of them (one 128-byte line each)
constexpr int kBigMapLayer = 1 << 20; // elements from which a full-map layer's bucket list goes through k_filter
// Candidate bound predicted from the thresholds of the two calls before, on a log2 scale: used
// while the threshold moved by at most kTrendMaxLog2 between those calls.
constexpr float kTrendMaxLog2 = 0.14f;         // a factor of 1.10 per call
constexpr float kMarginInitLog2 = 0.02f;       // safety margin below the lowest threshold expected (1.4 %)
constexpr float kMarginMaxLog2 = 0.25f;        // it doubles after every bound that lay too high, up to this
constexpr float kMarginDecay = 0.97f;          // per call, back towards the initial margin
constexpr float kMarginSafety = 1.5f;          // a forecast that came out too high by s widens the margin to 1.5 s + 0.01
constexpr uint32_t kCooldownCalls = 4;         // calls without a predicted bound after a failed one
// Candidate bounds lie between 2^-40 and 2^40 (float32 bit patterns): the main pass tests scores
// against them in float32, and its error bounds need that range.  A layer whose bound would fall
// outside (gradients of the order of 1e-12 or 1e12) is ranked on the full map.
constexpr uint32_t kPreF32MinKey = (127u - 40u) << 23;
constexpr uint32_t kPreF32MaxKey = (127u + 40u) << 23;
constexpr int kSamplingCalls = 10;             // first calls with a workspace: a layer without a predicted bound
                                               // takes one sampled from the call's own scores (later: the full map)

// Tile of the block-score kernel (block reading): kBlockTileRows block rows by
// block_tile_cols(p) block columns, i.e. 8p x (8 .. 256)p elements.
constexpr int kBlockTileRows = 8;
#if defined(__HIPCC__)
__host__ __device__
#endif
constexpr int block_tile_cols(int p) { return p == 1 ? 256 : p == 3 ? 64 : 32; }

// How the k_l-th largest score of a layer is found (per layer, decided on the device).
enum LayerMode : uint32_t {
    kModeCandidates = 0,  // scores above a sampled bound are recorded per tile; exact select on them
    kModeFullMap = 1,     // score map + histogram over every element (always exact, more traffic)
    kModeSkip = 2,        // k_l = 0: nothing is selected
};

// Sampled tiles of a layer: one tile in 2^shift, picked by a multiplicative hash of the
// tile's index inside the layer.  Larger layers are sampled more thinly (the estimate only
// needs a few hundred tiles); a layer of fewer than 128 tiles is "sampled" whole, so its bound
// comes from all of its scores.
#if defined(__HIPCC__)
__host__ __device__
#endif
inline bool tile_is_sampled(uint32_t local_tile, uint32_t shift) {
    return shift == 0u || ((local_tile * 2654435761u) >> (32u - shift)) == 0u;
}
inline uint32_t sample_shift(uint32_t n_tiles) {
    return n_tiles >= 16384u ? 6u : n_tiles >= 4096u ? 5u : n_tiles >= 128u ? 4u : 0u;
}

// One layer as the kernels see it.
struct LayerDev {
    int64_t elem_off;    // offset of the layer in the g / r / NSI arenas (elements)
    int64_t out_off;     // first pair of the layer in out_idx / out_val
    int64_t centre_off;  // first entry of the layer in out_centre_idx
    uint64_t list_off;   // first entry of the layer's threshold-bucket list
    uint64_t slot_off;   // first entry of the layer's tile slots (large layers)
    uint32_t R, C, G, k;
    uint32_t p, tiles_x, tile_begin, n_tiles;   // tile_begin: first tile inside its p-group launch
    uint32_t chunk_begin, n_chunks, cap, tile_begin_all;  // tile_begin_all: first tile over all layers
    uint32_t large;         // 1: eligible for the candidate path ("large layer" in the comments of this code: the
                            //    name is from when only layers of many tiles were; today the keep ratio decides)
    uint32_t group_begin;   // first slot group of the layer
    uint32_t n_groups;      // ceil(n_tiles / kSlotGroup)
    uint32_t hint_target;   // sampled scores wanted at or above the candidate bound
    uint32_t n_sampled;     // sampled tiles of the layer
    uint32_t list_cap;      // capacity of the threshold-bucket list
    uint32_t list_shards;   // shards the list is split into (each list_cap / list_shards entries, own counter)
    uint32_t slot_cap;      // entries per tile slot: kSlotCapMax, or what a tile of the layer can hold if that is less
    uint32_t cgroup_begin;  // first chunk group (kChunkGroup chunks) of the layer, numbered over all layers
    uint32_t pad_;
};
static_assert(sizeof(LayerDev) == 128, "LayerDev layout");

// Per-layer selection state (40 bytes), lives in the workspace, rewritten by every call.
struct SelState {
    unsigned long long T;   // threshold on the composite key (score bits << 32 | ~index)
    uint32_t k_rem;         // centres still to take inside the current bucket
    uint32_t done;          // threshold is final
    uint32_t mode;          // LayerMode
    uint32_t hint_key;      // candidate bound (score bits), candidate path only; 0: still to come from the sample
    uint32_t overflow;      // candidate path: a tile slot overflowed
    uint32_t lo;            // first ranking digit resolved: the k-th score lies in [lo, lo + 2^span)
    uint32_t span;
    uint32_t predicted;     // 1: the candidate bound was predicted from earlier calls, not sampled
};
static_assert(sizeof(SelState) == 40, "SelState layout");

// What a large layer remembers from one call to the next (uploaded as zeros with the tables).
struct PredState {
    uint32_t tau1;          // score bits of the last call's threshold (0: none yet)
    uint32_t tau2;          // ... and of the call before it
    float margin;           // safety margin below the predicted threshold, in log2 units (0: the initial one)
    uint32_t cooldown;      // calls left that take the sampled bound (after a failed bound)
    float forecast;         // log2 of the threshold this call was expected to end on, before the margin ...
    uint32_t has_forecast;  // ... when two earlier thresholds allowed one (also in calls that sample their bound)
};
static_assert(sizeof(PredState) == 24, "PredState layout");

// State of the cross-layer ranking of |w| (rsdgc_dynamic_ratios).
struct DynState {
    unsigned long long k_rem;   // weights still to take inside the current bucket
    uint32_t prefix;            // resolved high bits of the 31-bit key |w|
    uint32_t pad_;
};

// Directory entry used to map a workgroup id to a layer by binary search.
struct DirEntry {
    uint32_t begin;   // first tile / chunk / slot group of the layer
    uint32_t layer;
};

// A sampled tile: which layer, which tile inside it.
struct SampleEntry {
    uint32_t layer;
    uint32_t local_tile;
};

// Work item of the candidate passes: kSlotGroup (or fewer) consecutive tile slots of a large layer.
struct GroupEntry {
    uint32_t layer;
    uint32_t slot0;      // first tile slot (index over the tiles of all layers)
    uint32_t ntile;      // slots in the group
    uint32_t pad_;
};

// Work item of the score-map passes: one 8192-element chunk of a layer ranked on the full map.
struct ChunkEntry {
    uint32_t layer;
    uint32_t start;      // first element of the chunk inside the layer
    uint32_t len;        // elements in the chunk
    uint32_t pad_;
    uint64_t arena_off;  // elem_off + start
};

// Work item of the count pass: up to kCountChunks consecutive chunks of a layer (a quarter of a
// chunk group).
struct CountGroup {
    uint64_t word0;        // first 32-bit word of the group's mask bits
    uint32_t first_chunk;
    uint32_t n_chunks;
    uint32_t n_words;      // mask words of these chunks (a layer's last chunk may be short)
    uint32_t group;        // the chunk group (kChunkGroup chunks) they belong to
};
static_assert(sizeof(CountGroup) == 24, "CountGroup layout");

// Everything the 1-D passes need to know about one 8192-element chunk (one load instead of a
// chain chunk -> layer -> layer table).
struct ChunkInfo {
    uint64_t arena_off;  // elem_off + start
    uint64_t out_off;    // first pair of the chunk's layer in out_idx / out_val
    uint32_t layer;
    uint32_t start;      // first element of the chunk inside the layer
    uint32_t len;        // elements in the chunk
    uint32_t cap;        // capacity of the layer's output segment
    // for the chunk's prefix (kept elements of the layer before the chunk), which is the sum
    // of the totals of the layer's earlier chunk groups and of the earlier chunks of its own
    uint32_t group;              // chunk group (kChunkGroup chunks of one layer), numbered over all layers
    uint32_t group_first_chunk;  // first chunk of that group
    uint32_t layer_first_group;  // first group of the layer
    uint32_t last;               // 1: the layer's last chunk (it reports the layer's total)
    uint32_t gstride;            // words between two chunk-group counters: kGroupCntStride in a plan that counts
    uint32_t pad_;               // its kept elements where their bits are set (many adds per counter), else 1
};
static_assert(sizeof(ChunkInfo) == 56, "ChunkInfo layout");

// Byte offsets of the workspace sections (all multiples of 256).
struct WsLayout {
    // uploaded tables
    size_t layers = 0;       // LayerDev[n_layers]
    size_t tile_dir = 0;     // DirEntry[] per p-group, each closed by a sentinel
    size_t chunk_dir = 0;    // DirEntry[n_layers + 1]
    size_t large_dir = 0;    // DirEntry[] per p-group over its large layers, each closed by a sentinel
    size_t all_tile_dir = 0; // DirEntry[n_layers + 1]: tiles of all layers in layer order
    size_t samples = 0;      // SampleEntry[] per p-group
    size_t chunk_layer = 0;  // uint32[n_chunks]: layer of every 8192-element chunk
    size_t chunk_info = 0;   // ChunkInfo[n_chunks]
    size_t cand_groups = 0;  // GroupEntry[]: slot groups of the large layers (work list of the candidate passes)
    size_t map_chunks = 0;   // ChunkEntry[]: chunks of the other layers that select something
    size_t map_tiles = 0;    // SampleEntry[]: tiles of those layers
    size_t count_groups = 0; // CountGroup[n_count_groups]
    size_t pred = 0;         // PredState[n_layers]  uploaded as zeros, then kept by the kernels from call to call
    size_t table_bytes = 0;  // bytes uploaded from the host
    size_t state = 0;        // SelState[n_layers], rewritten at the start of every compress
    size_t flags = 0;        // uint32[64]  [0]: some large layer is ranked on the full map in this call (set at the
                             //             start of every compress, raised by the kernels that send a layer there)
    // cleared at the start of every compress
    size_t zero_begin = 0;
    size_t hist = 0;         // uint32[n_layers][kHistBins]  first ranking digit
    size_t hist_s = 0;       // uint32[n_layers][kHistBins]  sampled scores of the large layers (coarse digit)
    size_t hist1 = 0;        // uint32[n_layers][kLevel1Bins]  second ranking digit
    size_t chunk_cnt = 0;    // uint32[n_chunks]  kept elements per chunk
    size_t chunk_ccnt = 0;   // uint32[n_chunks]  selected centres per chunk
    size_t group_cnt = 0;    // uint32[n_chunk_groups * kGroupCntStride]  kept elements per chunk group, each counter on its own cache line
    size_t group_ccnt = 0;   // the same for the selected centres
    size_t list_cnt = 0;     // uint32[n_layers][kListShards][kListCntStride]  keys gathered per list shard
    size_t list2_cnt = 0;    // uint32[n_layers]  of those, keys that k_filter picked for k_finish
    size_t feed = 0;         // uint32[16][8][32]  work-feed counters of the NSI launches
    size_t mask = 0;         // uint32[total_elems / 32]  kept-element bitmask
    size_t cmask = 0;        // uint32[total_elems / 32]  selected-centre bitmask
    size_t zero_end = 0;
    // not cleared
    size_t slot_cnt = 0;     // uint32[n_tiles_all]  candidates recorded per tile
    size_t slot_ent = 0;     // uint64[sum over the layers of n_tiles * slot_cap]  their composite keys
    size_t list_ent = 0;     // uint64[sum list_cap]  composite keys of each layer's threshold bucket
    size_t list2_ent = 0;    // uint64[n_layers][2048]  keys sharing the first two digits (plans with big_map_layers)
    size_t nsi = 0;          // float[total_elems]  score map (full-map layers only)
    size_t dyn = 0;          // scratch of rsdgc_dynamic_ratios: DynState, uint64[kHistBins], uint32[2 * n_layers]
    size_t apply_ranges = 0; // uint32[RSDGC_MAX_MSGS][n_chunks][2]  rsdgc_apply: each message's pairs per chunk
    size_t total = 0;
};

struct PGroup {           // layers sharing one neighbourhood side: one launch per NSI pass
    int p = 0;
    uint32_t n_tiles = 0;
    uint32_t dir_begin = 0;     // index of the group's first DirEntry in tile_dir
    uint32_t dir_count = 0;     // entries excluding the sentinel
    uint32_t sample_begin = 0;  // index of the group's first SampleEntry: first every tile of the layers that are
    uint32_t n_map_samples = 0; // always ranked on the full map (n_map_samples entries), then the sampled tiles
    uint32_t n_samples = 0;     // of the others (n_samples entries in all)
    // the group's large layers only (the main pass and its fallback walk no other tiles, so
    // that equal shares of the walk are equal shares of the work)
    uint32_t large_dir_begin = 0;   // index of the first DirEntry in large_dir
    uint32_t large_dir_count = 0;   // entries excluding the sentinel
    uint32_t n_large_tiles = 0;
};

}  // namespace rsdgc

struct rsdgc_plan_s {
    int32_t n_layers = 0;
    double alpha = 0.5;
    std::vector<rsdgc_shape_t> shapes;
    std::vector<int32_t> p;
    std::vector<double> ratio;
    std::vector<rsdgc::LayerDev> layers;
    std::vector<rsdgc::PGroup> groups;
    std::vector<rsdgc::DirEntry> tile_dir;
    std::vector<rsdgc::DirEntry> chunk_dir;
    std::vector<rsdgc::DirEntry> all_tile_dir;
    std::vector<rsdgc::DirEntry> large_dir;
    std::vector<rsdgc::SampleEntry> samples;
    std::vector<rsdgc::GroupEntry> cand_groups;
    std::vector<rsdgc::ChunkEntry> map_chunks;
    std::vector<rsdgc::SampleEntry> map_tiles;
    uint32_t n_tiles_all = 0;
    uint64_t slot_entries = 0;          // composite keys in all tile slots together
    uint32_t n_slot_groups = 0;
    bool any_large = false;
    bool big_map_layers = false;        // some layer of a million elements or more is ranked on the full map
    int64_t total_elems = 0;
    int64_t out_capacity = 0;
    int64_t centre_capacity = 0;
    uint32_t n_chunks = 0;
    uint32_t n_chunk_groups = 0;  // chunk groups over all layers
    uint32_t n_count_groups = 0;  // work items of the count pass
    int work_feed = 0;            // RSDGC_FEED_*
    rsdgc::WsLayout ws;
    std::vector<unsigned char> table;   // host image of the uploaded tables
    // device-side bookkeeping
    uint64_t version = 1;               // bumped by set_ratios
    uint64_t serial = 0;                // unique per plan of this process (never reused, unlike its address)
    const void *uploaded_ws = nullptr;
    int calls_since_upload = 0;         // compress calls since the tables went to uploaded_ws (counted up to kSamplingCalls)
    uint64_t uploaded_version = 0;
    // block reading (non-overlapping p x p neighbourhoods): this plan describes the element
    // matrices; `inner` describes the block grids as layers with p = 1 and the same k_l, and
    // the selection machinery runs on it.  The workspace is this plan's tables followed by
    // inner's whole workspace.
    bool blocks = false;
    rsdgc_plan_s *inner = nullptr;
    std::vector<int64_t> k_override;    // inner plan only: k_l taken from the outer plan
    ~rsdgc_plan_s() { delete inner; }
    bool allow_candidates = true;       // false forces the full-map path for every layer
    // optional per-stage timing: (RSDGC_N_STAGES + 1) events per recorded call (hipEvent_t)
    std::vector<void *> prof_events;
    int prof_max_calls = 0;
    int prof_calls = 0;
};

namespace rsdgc {
// Host-only helpers implemented in rsdgc_plan.cpp.
int64_t keep_count(int64_t G, int p, double rho);   // Eq. 11
int build_tables(rsdgc_plan_s *plan);               // fills layers, dirs, ws, table
}  // namespace rsdgc
