// HIP kernels (gfx950, wave64) and the device-facing entry points of the C ABI.
//
// Pipeline of one rsdgc_compress call, all layers per launch.  "Candidate path": a layer whose
// keep ratio leaves room for it records only the centres whose score reaches a bound and ranks
// those; the other layers are ranked on a full score map.  The result is the same on both.
//   begin      zero histograms, bitmasks, counters, flags; per-layer state; for every layer on
//              the candidate path the bound predicted from the thresholds of the two calls before
//   first pass every tile of the layers that are always ranked on the full score map: v = r + g
//              (Eq. 12), NSI (Eqs. 6-10), score map, exact 12-bit histogram; during the first calls
//              with a workspace, in the same launch, one tile in 16 .. 64 of the candidate-path
//              layers that have no predicted bound: their score histogram gives a bound with
//              about 2 k_l centres expected above it (k_hint).  Not launched when it has no tiles.
//   capture    the main pass: v = r + g and NSI for every element of the candidate-path layers;
//              centres whose score reaches the bound are recorded per tile (no score map) and
//              counted in fine bins above the bound; with a second residual arena v is stored
//              there as it is formed
//   find0      first ranking digit of every layer; a layer whose bound caught fewer than k_l
//              centres, or overfilled a tile, falls back to the full map (a flag tells the
//              fallback kernels there is work)
//   fallback   score map + histogram of such layers (rare)
//   select     gather: the candidates above each layer's threshold bucket are selected for certain
//              and mark their windows; the bucket's keys are copied to a list and their next digit
//              counted; finish: one workgroup per layer resolves the remaining digits
//              (Algorithm 1's ranking; Eq. 11's k_l) and keeps the threshold for the next calls
//   mark       the bucket's keys that reach the threshold set the bits of their p x p window
//              (Section III-C: whole neighbourhoods are kept); full-map layers: every centre
//   count      kept elements per chunk and per group of chunks (no scan kernel: each consumer
//              adds up its own prefix from those)
//   emit       ordered (index, value) pairs and the residual update (Eq. 12): either only the
//              kept elements are touched (second arena), or g and r are streamed again
//              (update in place)
//
// Sections of this file, in order (each starts with a "// ---- name --" line):
//   begin            k_begin
//   work feed        WorkFeed: tiles handed to persistent workgroups through per-XCD counters
//   nsi              k_nsi<P, PASS, MOM, FEED>: the four NSI passes, with or without Eq. 12's momentum
//   ranking digits   block_find_digit, publish_threshold
//   hint .. finish   k_hint, k_find0, k_gather, k_filter, k_finish: bounds and the radix select
//   mark             k_mark: p x p windows into the bitmask
//   count            k_count, chunk_prefix_wave0
//   emit             k_emit, k_emit_sparse, k_emit_centres
//   decompress       k_zero_layers, k_scatter
//   block reading    k_block_nsi, k_emit_blocks, k_scatter_blocks
//   apply            k_apply_ranges, k_apply_chunks, k_apply_single, k_apply_blocks (receiving side)
//   dynamic ratios   k_dyn_*
//   host side        launch helpers and the extern "C" entry points
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "rsdgc_internal.h"

using namespace rsdgc;

namespace {

thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e, const char *what) {
    std::snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
    return RSDGC_EHIP;
}
#define HIP_TRY(expr)                                        \
    do {                                                     \
        hipError_t e_ = (expr);                              \
        if (e_ != hipSuccess) return hip_fail(e_, #expr);    \
    } while (0)

// Composite ranking key  K = (score bits << 32) | ~index.  Scores are non-negative floats, so
// their bit pattern orders like the value; ~index makes the lower index the larger key; all
// keys of a layer are distinct.
constexpr uint32_t kNumCUs = 256;   // MI355X
__device__ __forceinline__ unsigned long long composite_key(uint32_t score_bits, uint32_t index) {
    return (static_cast<unsigned long long>(score_bits & 0x7fffffffu) << 32) |
           static_cast<unsigned long long>(~index);
}

// Entry e with dir[e].begin <= id < dir[e + 1].begin  (dir has n entries + a sentinel).
__device__ __forceinline__ uint32_t dir_lookup(const DirEntry *__restrict__ dir, uint32_t n,
                                               uint32_t id) {
    uint32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (dir[mid].begin <= id) lo = mid; else hi = mid;
    }
    return lo;
}

// The same from entry e, which lies at or before the wanted one: a workgroup's next item is often in
// the same layer or the next, but in a plan of many small layers it may lie hundreds of layers on --
// stepping there entry by entry is a chain of dependent loads that costs more than the tile itself.
__device__ __forceinline__ uint32_t dir_advance(const DirEntry *__restrict__ dir, uint32_t n, uint32_t e,
                                                uint32_t id) {
    if (id < dir[e + 1].begin) return e;
    ++e;
    if (id < dir[e + 1].begin) return e;
    return e + 1 + dir_lookup(dir + e + 1, n - (e + 1), id);    // (id < dir[n].begin, so e + 1 < n)
}

// Workgroups are handed to the 8 XCDs round-robin by id; give each XCD one contiguous
// range of tiles so that neighbouring tiles (which share halo rows/columns) meet in
// the same L2.
__device__ __forceinline__ uint32_t xcd_contiguous(uint32_t bid, uint32_t n) {
    const uint32_t xcd = bid & 7u, slot = bid >> 3;
    const uint32_t per = n >> 3, rem = n & 7u;
    return xcd * per + (xcd < rem ? xcd : rem) + slot;
}

// Inclusive scan over the NW * 64 threads of a workgroup.
template <int NW>
__device__ __forceinline__ uint32_t block_scan_incl_n(uint32_t v, uint32_t *wave_tot /*[NW]*/) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    if (lane == 63) wave_tot[wave] = v;
    __syncthreads();
    uint32_t add = 0;
#pragma unroll
    for (int w = 0; w < NW - 1; ++w)
        if (w < wave) add += wave_tot[w];
    const uint32_t r = v + add;
    __syncthreads();   // wave_tot may be reused by the caller
    return r;
}

// Position for one appended item per flagged lane: one atomic on the LDS counter per wave.
// Called by all 64 lanes of a wave; the result is meaningful for flagged lanes only.
__device__ __forceinline__ uint32_t wave_append(uint32_t *counter, bool flag) {
    const unsigned long long m = __ballot(flag);
    if (m == 0ull) return 0u;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t leader = static_cast<uint32_t>(__ffsll(static_cast<long long>(m))) - 1u;
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(counter, static_cast<uint32_t>(__popcll(m)));
    base = __shfl(base, static_cast<int>(leader), 64);
    return base + static_cast<uint32_t>(__popcll(m & ((1ull << lane) - 1ull)));
}

// Inclusive scan over the 256 threads of a workgroup (4 waves of 64).
__device__ __forceinline__ uint32_t block_scan_incl(uint32_t v, uint32_t *wave_tot /*[4]*/) {
    return block_scan_incl_n<4>(v, wave_tot);
}

// Safety margin (in log2 of the score) of a layer's first predicted bounds: the k-th largest of few
// scores moves more from call to call than that of many.
__device__ __forceinline__ float margin_init_log2(uint32_t k) {
    return fmaxf(kMarginInitLog2, 0.75f * rsqrtf(static_cast<float>(max(k, 1u))));
}

// ---------------------------------------------------------------- begin --
// Start of a compress call: all workgroups but the last clear the histograms, counters and
// bitmasks; the last one writes every layer's initial selection state.  A large layer gets its
// candidate bound here when the thresholds of its last two calls (kept in `pred`) lie close
// together.  While a residual builds up, the threshold keeps moving in one direction by steps
// that, on a logarithmic scale, shrink smoothly from call to call; so after a step d of
// log2(threshold) the next one is taken to lie between 0.6 d and 1.15 d, and the bound sits a
// margin below the lowest threshold that allows.  The margin doubles after a bound that lay too high
// and halves after one that lay too low (k_find0).
// The result of the call never depends on the bound -- only whether the layer has to be redone
// through the full map.  Without a usable history (first calls, after a failure, a threshold
// that jumps) the bound comes from a sample of this call's scores (k_hint) during the first
// calls with a workspace (`sampling`); later such a layer is ranked on the full map until its
// threshold has settled, and the call needs neither the sampled tiles nor k_hint.
// flags[0] tells the fallback kernels whether any large layer is on the full map.
__global__ __launch_bounds__(256) void k_begin(uint4 *__restrict__ p, size_t n16,
                                               const LayerDev *__restrict__ layers,
                                               SelState *__restrict__ state, int n_layers,
                                               PredState *__restrict__ pred /* nullable */,
                                               uint32_t *__restrict__ flags, int sampling) {
    if (blockIdx.x + 1 == gridDim.x) {
        bool fallback_work = false;
        for (int l = threadIdx.x; l < n_layers; l += 256) {
            SelState s;
            const LayerDev L = layers[l];
            s.T = L.k == 0 ? ~0ull : 0ull;   // no key reaches ~0: nothing is selected when k = 0
            s.k_rem = L.k;
            s.done = L.k == 0 ? 1u : 0u;
            s.mode = L.k == 0 ? kModeSkip : (L.large ? kModeCandidates : kModeFullMap);
            s.hint_key = 0;
            s.overflow = 0;
            s.lo = 0;
            s.span = 0;
            s.predicted = 0;
            if (pred && s.mode == kModeCandidates) {
                PredState ps = pred[l];
                // after a failed bound the layer goes back to sampled bounds for a few calls -- where there
                // are any: past the calls that sample, the alternative would be the full map, and the
                // widened margin is tried at once
                const bool paused = ps.cooldown > 0 && sampling;
                // the call before failed: its threshold was a jump, not part of a trend -- the forecast
                // is that threshold itself
                const bool just_failed = ps.cooldown == kCooldownCalls;
                if (ps.cooldown > 0) ps.cooldown -= 1;
                ps.has_forecast = 0;
                if (ps.tau1 >= (1u << 23) && ps.tau2 >= (1u << 23)) {   // (both in the normal float32 range)
                    const float l1 = __log2f(__uint_as_float(ps.tau1)), l2 = __log2f(__uint_as_float(ps.tau2));
                    const float d = l1 - l2;
                    const float dd = just_failed ? 0.f : fminf(fmaxf(d, -2.f * kTrendMaxLog2), kTrendMaxLog2);
                    // the forecast is made in every call, used or not: how far the threshold then ends
                    // below it is what sizes the margin (publish_threshold)
                    ps.forecast = l1 + (dd > 0.f ? 0.6f * dd : 1.15f * dd);
                    ps.has_forecast = 1;
                    // (a threshold that jumps: sampled bounds while there are any; later the trend is
                    // taken as far as it is trusted -- a bound that fails costs less than the full map)
                    if (!paused && (fabsf(d) <= kTrendMaxLog2 || !sampling)) {   // (d, not dd: a jump is sampled)
                        const float margin = ps.margin > 0.f ? ps.margin : margin_init_log2(L.k);
                        const float bound = exp2f(ps.forecast - margin);
                        const uint32_t key = __float_as_uint(bound);
                        if (key >= kPreF32MinKey && key <= kPreF32MaxKey) {   // (else: no bound, the full map)
                            s.hint_key = key;
                            s.predicted = 1;
                        }
                    }
                }
                pred[l] = ps;
                if (!s.predicted && !sampling) {
                    s.mode = kModeFullMap;
                    fallback_work = true;
                }
            }
            state[l] = s;
        }
        const int any = __syncthreads_or(fallback_work ? 1 : 0);
        if (threadIdx.x == 0) flags[0] = any ? 1u : 0u;
        return;
    }
    const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x - 1) * 256;
    for (size_t j = i; j < n16; j += stride) p[j] = make_uint4(0, 0, 0, 0);
}

// 16-byte store of data this call does not read again (the new residual / momentum arena):
// marked non-temporal so that it does not displace the halo rows and candidate slots that
// later tiles and kernels find in cache (measured: -12 us on the VGG-19 main pass).
__device__ __forceinline__ void store_streaming(float *__restrict__ dst, const float4 v) {
    typedef float vf4 __attribute__((ext_vector_type(4)));
    const vf4 vv = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(vv, reinterpret_cast<vf4 *>(dst));
}

// 16-byte load of data no other workgroup reads and this one reads once: marked non-temporal,
// so that it does not displace what is reused (measured: -8 % on the block-score pass).
__device__ __forceinline__ float4 load_streaming(const float *__restrict__ src) {
    typedef float vf4 __attribute__((ext_vector_type(4)));
    const vf4 t = __builtin_nontemporal_load(reinterpret_cast<const vf4 *>(src));
    return make_float4(t.x, t.y, t.z, t.w);
}

// A float that is the same in every lane, moved to a scalar register.
__device__ __forceinline__ float uniform_f32(float x) {
    return __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(x)));
}

// Eqs. 8-10 from the window sums sa = sum|w|, ss = sum w, sq = sum w^2 (n = p*p slots):
//   mean = sa / n,  std = sqrt(d) / n  with  d = n*sq - ss^2 = n^2 * variance,
//   NSI = alpha*mean + (1-alpha)*std = ca*sa + cb*sqrt(d).
// d is formed from two separately rounded products.  That form cancels: its absolute error
// is a few 1e-16 of n*sq, so the relative error of the standard deviation grows like
// 1e-16 * (1 + mean^2 / variance).  A window whose d falls below kCancelFrac * n*sq
// (|mean| beyond a thousand standard deviations: near-constant values on a large offset)
// is therefore evaluated again the way Eq. 10 is printed -- window_ssd below -- and only the
// others (relative error of the one-pass form below 3e-9) keep the one-pass value.
constexpr double kCancelFrac = 1.0 / 1048576.0;

// The main pass rules out the centres below the bound in float32 (half the registers of the same
// test in double, no conversions).  It must never rule out a centre that
// the evaluation in full would record, so every float32 quantity is bounded against the exact one.
// With u = 2^-24, n = p*p, exact window sums SA = sum|w|, SS = sum w, SQ = sum w^2, D = n SQ - SS^2
// (SA^2 <= n SQ, |SS| <= SA), and a bound B in [2^-40, 2^40] (nothing of weight under- or overflows):
//   sa = SA (1 + t), |t| <= (n-1) u          (non-negative terms)
//   n sq - ss^2 differs from D by at most (3n + 3) u * n SQ: n u from the roundings of sq and of the
//     product with n, 2n u from ss (off by at most (n-1) u SA) squared, the rest from the last fma;
//     d_hi = that + kSlack * n sq with kSlack = 1.3 (3n + 3) u is therefore at least D;
//   rest = B' - ca sa with B' = B * kBoundFactor = B (1 - 2^-22 - 2.04 n u), rounded down: at most the exact
//     B (1 - 2^-22) - ca SA whenever ca SA < 2 B, and negative otherwise;
//   the centre stays unless rest > 0 and cb^2 d_hi < rest^2 (1 - 1e-6): the seven roundings between
//     the two sides change their ratio by less than 8 u < 1e-6.
// The comparison is written so that a NaN on either side keeps the centre, and an infinite sum does:
// such windows are left to the evaluation in full.  Squares of values below 2^-63 underflow; what is
// lost (below 2^-126 each) is far less than either slack for a bound of at least 2^-40.  Outside
// that range no bound is handed out: the layer is ranked on the full map (k_begin, k_hint).
template <int P> struct PreF32 {
    static constexpr float kSlack = 1.3f * (3.f * P * P + 3.f) * 5.9604645e-8f;
    static constexpr double kBoundFactor = 1.0 - 1.0 / 4194304.0 - 2.04 * (P * P) * 5.9604645e-8;
};

constexpr int kQueueCap = 1024;      // centres one tile can queue for full evaluation (twice the largest slot)

__device__ __forceinline__ double var_n2_one_pass(double ss, double nsq) {
    return __dsub_rn(nsq, __dmul_rn(ss, ss));
}

// Eq. 10 as printed, for the rare window where the one-pass form cancels: the sum over the
// P x P window at `win` (LDS, row pitch `pitch`) of (w - m)^2, rows top to bottom, left to right.
// Equal windows give equal bits wherever they lie, and a constant window gives exactly 0
// (m = P*P*c / (P*P) is exact), which the ranking's tie rule relies on.  Loops are kept rolled:
// this is cold code inside an unrolled loop.
template <int P>
__device__ __forceinline__ double window_ssd(const float *win, int pitch, double m) {
    double acc = 0.0;
#pragma unroll 1
    for (int dx = 0; dx < P; ++dx) {
#pragma unroll 1
        for (int dy = 0; dy < P; ++dy) {
            const double e = static_cast<double>(win[dx * pitch + dy]) - m;
            acc += __dmul_rn(e, e);
        }
    }
    return acc;
}

// ca*sa + cb*sqrt(d).  The square root is one v_rsq_f64 seed, one coupled Newton step and one
// residual correction (about 1 ulp in double); the floor 1e-300 stands in for 0 and vanishes
// when the score is rounded to float32.
__device__ __forceinline__ double nsi_from_var(double sa, double d, double ca, double cb) {
    d = fmax(d, 1e-300);
    const double y = __builtin_amdgcn_rsq(d);
    double g = d * y, h = 0.5 * y;
    const double r = fma(-h, g, 0.5);
    g = fma(g, r, g);
    h = fma(h, r, h);
    const double e = fma(-g, g, d);
    g = fma(e, h, g);
    return fma(cb, g, ca * sa);
}

// ----------------------------------------------------------- work feed --
// Hands the items of a launch (tiles) to its persistent workgroups.  With a fixed strided
// share per workgroup the workgroups drift apart (measured on the VGG-19 main pass: the first
// leaves at 240 us, the mean at 310, the last at 390); here every workgroup takes its next item
// from a counter when it is ready.
//
// Locality is kept: the items are cut into stretches of 8 * S consecutive items, part d of
// every stretch belongs to domain d (one per XCD: workgroups are handed to the XCDs
// round-robin by id), and a domain's counter walks its parts in order -- so at any moment an
// XCD's workgroups hold consecutive items (neighbouring tiles share halo rows in that XCD's
// L2), and a counter's cache line stays in that XCD's L2.  A workgroup leaves when its own
// domain is used up: taking from other domains was measured too (in ring order, or from the
// fullest), and the tickets it costs on other XCDs' counters outweigh the better balance.
//
// The ticket for the item after the current one is requested (one atomic by thread 0) when the
// current item starts and read when it ends, so its latency is hidden.
constexpr uint32_t kNoItem = 0xffffffffu;
constexpr int kFeedDomains = 8;
constexpr int kFeedStride = 32;          // uint32 between two counters (one 128-byte line each)
constexpr int kFeedSets = 16;            // counter sets per call: (pass, p-group) pairs

// Items of domain d: part d of every full stretch, and its share of the last, partial one.
__device__ __forceinline__ uint32_t feed_domain_items(uint32_t n_items, uint32_t shift, uint32_t d) {
    const uint32_t S = 1u << shift;
    const uint32_t full = n_items >> (shift + 3), rem = n_items & ((S << 3) - 1u);
    const uint32_t lo = d << shift;
    return (full << shift) + (rem > lo ? min(rem - lo, S) : 0u);
}

struct WorkFeed {
    uint32_t *ctr;        // the workgroup's domain counter (zero at launch)
    uint32_t items;       // items of that domain
    uint32_t shift, dom;
    uint32_t par;         // LDS slot of the next hand-over
    bool stashed;         // the requested ticket is already in that slot
    uint32_t pending;     // thread 0: the ticket requested last
    // (plain members whose values the compiler can follow through the loop: with the flags
    // packed into one word the main pass needed 15 more registers)

    // Thread 0 puts the requested ticket into LDS.  Reading it waits for the wave's memory
    // operations up to the request, and the compiler may make that a wait for everything
    // issued since.  So the item's code calls this after its loads have arrived and before
    // its first store; next() does it for items that never got there.
    __device__ __forceinline__ void stash(uint32_t *slot /*[2], LDS*/) {
        if (!stashed && threadIdx.x == 0) slot[par] = pending;
        stashed = true;
    }
    // Called by all threads of the workgroup (it contains a barrier); returns the next item or
    // kNoItem.
    __device__ __forceinline__ uint32_t next(uint32_t *slot) {
        if (!stashed && threadIdx.x == 0) slot[par] = pending;
        stashed = false;
        __syncthreads();
        const uint32_t t = __builtin_amdgcn_readfirstlane(slot[par]);   // the same in every lane: keep it scalar
        par ^= 1u;
        if (t >= items) return kNoItem;                 // uniform: the domain is used up
        if (threadIdx.x == 0) pending = atomicAdd(ctr, 1u);
        return ((t >> shift) * kFeedDomains + dom) * (1u << shift) + (t & ((1u << shift) - 1u));
    }
    // counters: the launch's kFeedDomains counters; log2_part: log2 S.
    __device__ __forceinline__ uint32_t first(uint32_t *__restrict__ counters, uint32_t n_items, uint32_t log2_part,
                                              uint32_t *slot) {
        dom = blockIdx.x % kFeedDomains;                // workgroups go to the XCDs round-robin by id
        shift = log2_part;
        items = feed_domain_items(n_items, shift, dom);
        ctr = counters + dom * kFeedStride;
        par = 0;
        stashed = false;
        pending = kNoItem;                              // an empty domain never touches its counter
        if (threadIdx.x == 0 && items != 0u) pending = atomicAdd(ctr, 1u);
        return next(slot);
    }
};

// ------------------------------------------------------------------ nsi --
// What one launch of the NSI kernel produces.
enum NsiPass : int {
    kPassMapOnly = 0,   // score map to a caller buffer (rsdgc_nsi)
    kPassFullMap = 1,   // score map + 12-bit histogram of the large layers that fell back to the full map
    kPassCapture = 2,   // candidates (score >= bound) recorded per tile, layers in candidate mode
    kPassSample = 3,    // first pass over the plan's tile list: 12-bit histogram of the sampled tiles
                        // of the large layers; score map + histogram of every tile of the others
};

struct NsiArgs {
    const LayerDev *layers;
    const DirEntry *dir;          // tile directory of the launch (all but kPassSample)
    uint32_t n_dir;
    uint32_t n_tiles;
    const SampleEntry *samples;   // kPassSample
    const float *grad;
    const float *resid;           // nullable: all-zero residual
    float *nsi_out;               // score map (kPassMapOnly, kPassFullMap)
    float *v_out;                 // nullable: second residual arena that receives v = r + g
    const float *mom;             // nullable: momentum arena u (Eq. 12, first line); then v = r + (m*u + g)
    float *mom_out;               // with mom: receives m*u + g wherever v_out receives v
    float m;                      // momentum factor
    const uint32_t *flags;        // [0] != 0: some large layer fell back to the full map
    uint32_t *hist;               // [n_layers][kHistBins]
    uint32_t *hist_s;             // [n_layers][kHistBins]  scores of the sampled tiles of the large layers
    const SelState *state;
    SelState *state_rw;           // same array; the main pass sets the overflow flag
    uint32_t *slot_cnt;           // [n_tiles_all]
    unsigned long long *slot_ent; // per large layer n_tiles slots of slot_cap entries, from the layer's slot_off
    double ca, cb;                // alpha / p^2, (1 - alpha) / p^2: NSI = ca * sum|w| + cb * sqrt(p^2 * sum w^2 - (sum w)^2)
    uint32_t *feed;               // work-feed counters of this launch (all but kPassMapOnly)
    uint32_t feed_shift;          // log2 of the items per domain and stretch
};

// Bucket that holds the k-th largest entry of a 4096-bucket histogram h (completed by an earlier
// launch), walking down from the top bucket.  One wave; every lane returns the same result
// (found = 0 when the histogram holds fewer than k entries).  Cold code inside hot kernels: its
// loops stay rolled so that it needs next to no registers.
struct WaveBucket {
    uint32_t bucket, above, count, found;
};
__device__ __forceinline__ WaveBucket wave_find_bucket(const uint32_t *__restrict__ h, uint32_t k) {
    const int lane = threadIdx.x & 63;
    constexpr int per = kHistBins / 64;
    const int hi = kHistBins - lane * per;              // lane 0 holds the top buckets
    uint32_t own = 0;
#pragma unroll 1
    for (int b = hi - 1; b >= hi - per; --b) own += h[b];
    uint32_t incl = own;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    const uint32_t excl = incl - own;
    WaveBucket r = {0u, 0u, 0u, 0u};
    const bool mine = excl < k && k <= incl;
    if (mine) {
        uint32_t acc = excl;
#pragma unroll 1
        for (int b = hi - 1; b >= hi - per; --b) {
            const uint32_t c = h[b];
            if (acc + c >= k) {
                r.bucket = static_cast<uint32_t>(b);
                r.above = acc;
                r.count = c;
                break;
            }
            acc += c;
        }
    }
    const unsigned long long who = __ballot(mine);
    if (who == 0ull) return r;
    const int src = __ffsll(static_cast<long long>(who)) - 1;
    r.bucket = __shfl(r.bucket, src, 64);
    r.above = __shfl(r.above, src, 64);
    r.count = __shfl(r.count, src, 64);
    r.found = 1u;
    return r;
}

// Work unit: one 16 x 256 tile of one layer.  The tile of v = r + g plus a halo of
// h = (P-1)/2 rows and 4 columns (16-byte aligned) goes to LDS; each thread then walks
// down the 16 rows of one column, keeping per-row horizontal sums of |w|, w and w^2
// for the last P rows in registers.  Every score that is stored, counted or recorded is
// computed in double: the variance as (P^2 * sum w^2 - (sum w)^2) / P^4, or -- where that
// form cancels -- from the tile again as Eq. 10 prints it; either way equal windows get
// equal scores wherever they lie and a constant window gets a variance of exactly 0.  The
// main pass (capture) runs the sweep in float32 instead and only decides there which centres
// cannot reach the layer's bound (PreF32 above); the others it evaluates in double as said.
// The capture variants are held to five waves per SIMD for p <= 3 and four for p = 5, 7
// (what their registers allow without spilling; measured faster than one wave less).
//
// A workgroup takes tiles b, b + W, ... of the launch (W workgroups, laid out so that each XCD
// gets one contiguous part of every stretch of W tiles: neighbouring tiles share halo rows in
// one L2), or -- FEED -- whatever the launch's work feed hands it next.  Its LDS histogram is
// flushed to the layer's global histogram only when the layer changes or its tiles end, so
// a launch issues few same-address global atomics.
// MOM: with Eq. 12's momentum term (a.mom, a.mom_out, a.m).  FEED: the workgroups take their
// tiles from the launch's work feed instead of a fixed strided share.
template <int P, int PASS, bool MOM, bool FEED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(PASS == kPassCapture && !MOM ? (P <= 3 ? 5 : 4) : 1, 8)))
void k_nsi(const NsiArgs a) {
    constexpr int H = (P - 1) / 2;
    constexpr int ROWS = kTileRows + 2 * H;
    constexpr int PADL = 4;
    constexpr int PITCH = kTileCols + 2 * PADL;   // 264 floats
    // One column per thread (two adjacent columns would share LDS reads, but the second set of row
    // sums costs 18 registers and a wave per SIMD).
    constexpr int RPT = kTileRows * kTileCols / 256;           // output rows per thread
    constexpr bool MAP = PASS == kPassMapOnly || PASS == kPassFullMap;
    constexpr bool CAPTURE = PASS == kPassCapture;
    constexpr bool FULLHIST = PASS == kPassFullMap || PASS == kPassSample;
    constexpr bool STORE_V = PASS != kPassMapOnly;
    constexpr int NBINS = FULLHIST ? kHistBins : (CAPTURE ? kFineBins : 1);
    __shared__ __attribute__((aligned(16))) float tile[ROWS * PITCH];
    __shared__ uint32_t lhist[NBINS];
    __shared__ unsigned long long cand[CAPTURE ? kSlotCapMax : 1];
    __shared__ uint16_t queue[CAPTURE ? kQueueCap : 1];
    __shared__ uint32_t ncand, nqueue;
    __shared__ uint32_t feed_slot[2];

    const int tid = threadIdx.x;
    // the launch's work items (tiles, or sampled tiles): at any moment the resident workgroups
    // work on one compact stretch of tiles, so neighbouring tiles' halo rows are still in
    // cache; inside a stretch each XCD takes one contiguous part
    const uint32_t n_items = a.n_tiles;
    const uint32_t stride = gridDim.x;
    if (PASS == kPassFullMap && a.flags[0] == 0u) return;   // no layer fell back: nothing to do
    WorkFeed feed;
    uint32_t first;
    if (FEED) {
        first = feed.first(a.feed, n_items, a.feed_shift, feed_slot);
        if (first == kNoItem) return;      // uniform
    } else {
        first = xcd_contiguous(blockIdx.x, gridDim.x);
        if (first >= n_items) return;
    }

    if (NBINS > 1)
        for (int b = tid; b < NBINS; b += 256) lhist[b] = 0;
    if (CAPTURE && tid == 0) { ncand = 0; nqueue = 0; }
    __syncthreads();

    uint32_t e = 0;                       // directory entry of the current layer
    if (PASS != kPassSample) e = dir_lookup(a.dir, a.n_dir, first);
    uint32_t cur_l = 0xffffffffu;         // layer whose counts sit in lhist
    uint32_t hint_key = 0;
    uint32_t *hist_base = a.hist;         // first pass: a.hist_s for the sampled tiles of a large layer
    bool active = true;
    bool whole = true;                    // every tile of the layer is visited: v and the scores go out
    LayerDev L;

    const double n = static_cast<double>(P * P);
    // (kernel arguments: the same in every lane, so they stay in scalar registers -- the scalar unit
    // has no floating point, a uniform value computed here would occupy vector registers)
    const double ca = a.ca, cb = a.cb;
    const float caf = uniform_f32(static_cast<float>(ca)), cb2f = uniform_f32(static_cast<float>(cb * cb));
    float bound_lof = 0.f;                // capture: a conservative form of the candidate bound (PreF32)
    static_assert(kTileCols * (kTileRows / RPT) == 256, "one thread per RPT rows of one column");
    const int c0 = tid % kTileCols, ty = tid / kTileCols;
    const int row_base = ty * RPT;

    for (uint32_t t = first; FEED ? t != kNoItem : t < n_items; t = FEED ? feed.next(feed_slot) : t + stride) {
        uint32_t l, local;
        if (PASS == kPassSample) {
            const SampleEntry se = a.samples[t];
            l = se.layer;
            local = se.local_tile;
        } else {
            e = dir_advance(a.dir, a.n_dir, e, t);
            l = a.dir[e].layer;
            local = t - a.dir[e].begin;
        }
        if (l != cur_l) {
            if (NBINS > 1 && cur_l != 0xffffffffu && active) {   // flush the finished layer's counts
                uint32_t *__restrict__ gh = hist_base + static_cast<size_t>(cur_l) * kHistBins;
                for (int b = tid; b < NBINS; b += 256) {
                    const uint32_t c = lhist[b];
                    if (c) { atomicAdd(&gh[b], c); lhist[b] = 0; }
                }
                __syncthreads();
            }
            cur_l = l;
            L = a.layers[l];
            active = true;
            hint_key = 0;
            whole = PASS != kPassSample || L.large == 0u;
            if (PASS == kPassFullMap || PASS == kPassCapture || (PASS == kPassSample && !whole)) {
                const SelState st = a.state[l];
                if (PASS == kPassFullMap) active = st.mode == kModeFullMap && L.large != 0u;
                else if (PASS == kPassSample) active = st.mode == kModeCandidates && st.hint_key == 0u;   // no predicted bound
                else active = st.mode == kModeCandidates;
                if (CAPTURE) {
                    hint_key = st.hint_key;
                    bound_lof = uniform_f32(__double2float_rd(static_cast<double>(__uint_as_float(hint_key)) * PreF32<P>::kBoundFactor));
                    // (k_begin and k_hint give no bound outside the range of the float32 test; should one
                    // arrive all the same, the layer is not captured and k_find0 sends it to the full map)
                    if (active && (hint_key < kPreF32MinKey || hint_key > kPreF32MaxKey)) {
                        active = false;
                        if (tid == 0 && hint_key != 0u) a.state_rw[l].overflow = 1u;
                    }
                }
            }
            if (PASS == kPassSample) hist_base = whole ? a.hist : a.hist_s;
        }
        if (!active) {                    // skip the rest of this layer
            if (!FEED && PASS != kPassSample) {
                const uint32_t nb = a.dir[e + 1].begin;          // first tile of the next layer
                t += (nb - t + stride - 1) / stride * stride - stride;   // loop increment adds the last stride
            }
            continue;
        }

        const int trow = static_cast<int>(local / L.tiles_x);
        const int tcol = static_cast<int>(local - static_cast<uint32_t>(trow) * L.tiles_x);
        const int R = static_cast<int>(L.R), C = static_cast<int>(L.C);
        const int x0 = trow * kTileRows, y0 = tcol * kTileCols;
        const float *__restrict__ g = a.grad + L.elem_off;
        const float *__restrict__ r = a.resid ? a.resid + L.elem_off : nullptr;

        // ---- load v = r + g for the tile and its halo; zero outside the matrix
        if ((C & 3) == 0) {
            // The tile's own 256 columns: wave w takes rows w, w + 4, ... of the tile and its row
            // halo, lane j the 16 bytes at column 4 j -- 1 KB per wave and row, and next to no
            // index arithmetic (a flat split of the tile into 16-byte pieces needs a division per
            // piece, which the compiler computes once and then keeps in a dozen registers).  The
            // column halo, H floats on either side of every row, is loaded as single floats by the
            // first 2 H ROWS threads.
            constexpr int ITER = (ROWS + 3) / 4;
            const int wave = tid >> 6, lane = tid & 63;
            const int ym = y0 + 4 * lane;
            const int hrow = H > 0 ? tid / (2 * H > 0 ? 2 * H : 1) : 0;
            const int hc = H > 0 ? tid - hrow * 2 * H : 0;              // 0 .. H-1 left of the tile, H .. 2H-1 right of it
            const int hy = hc < H ? y0 - 1 - hc : y0 + kTileCols + (hc - H);
            const int hx = x0 - H + hrow;
            const bool halo_thread = H > 0 && tid < 2 * H * ROWS;
            const bool halo_in = halo_thread && hx >= 0 && hx < R && hy >= 0 && hy < C;
            const size_t hoff = halo_in ? static_cast<size_t>(hx) * C + hy : 0;
            float4 gv[ITER], rv[ITER];
            float gh = 0.f, rh = 0.f;
#pragma unroll
            for (int it = 0; it < ITER; ++it) {
                const int rr = 4 * it + wave;
                const int x = x0 - H + rr;
                gv[it] = make_float4(0.f, 0.f, 0.f, 0.f);
                rv[it] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (rr < ROWS && x >= 0 && x < R && ym < C) {
                    const size_t off = static_cast<size_t>(x) * C + ym;
                    gv[it] = *reinterpret_cast<const float4 *>(g + off);
                    if (r) rv[it] = *reinterpret_cast<const float4 *>(r + off);
                }
            }
            if (halo_in) {
                gh = g[hoff];
                if (r) rh = r[hoff];
            }
            if (MOM) {                    // Eq. 12, first line: the gradient term becomes u = m*u + g
                const float *__restrict__ u = a.mom + L.elem_off;
                float4 uv[ITER];
                float uh = 0.f;
#pragma unroll
                for (int it = 0; it < ITER; ++it) {
                    const int rr = 4 * it + wave;
                    const int x = x0 - H + rr;
                    uv[it] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (rr < ROWS && x >= 0 && x < R && ym < C)
                        uv[it] = *reinterpret_cast<const float4 *>(u + static_cast<size_t>(x) * C + ym);
                }
                if (halo_in) uh = u[hoff];
                if (FEED) feed.stash(feed_slot);   // the loads are out, no store of this tile yet
                gh = __fmul_rn(a.m, uh) + gh;
#pragma unroll
                for (int it = 0; it < ITER; ++it) {
                    gv[it].x = __fmul_rn(a.m, uv[it].x) + gv[it].x;
                    gv[it].y = __fmul_rn(a.m, uv[it].y) + gv[it].y;
                    gv[it].z = __fmul_rn(a.m, uv[it].z) + gv[it].z;
                    gv[it].w = __fmul_rn(a.m, uv[it].w) + gv[it].w;
                    if (STORE_V && a.mom_out && whole) {   // the tile's own elements (not the halo) go out once
                        const int rr = 4 * it + wave;
                        const int x = x0 - H + rr;
                        if (rr >= H && rr < H + kTileRows && x < R && ym < C)
                            store_streaming(a.mom_out + L.elem_off + static_cast<size_t>(x) * C + ym, gv[it]);
                    }
                }
            }
            if (FEED) feed.stash(feed_slot);       // the loads are out, no store of this tile yet
#pragma unroll
            for (int it = 0; it < ITER; ++it) {
                const int rr = 4 * it + wave;
                if (rr < ROWS) {
                    float4 v;
                    v.x = rv[it].x + gv[it].x;
                    v.y = rv[it].y + gv[it].y;
                    v.z = rv[it].z + gv[it].z;
                    v.w = rv[it].w + gv[it].w;
                    *reinterpret_cast<float4 *>(&tile[rr * PITCH + PADL + 4 * lane]) = v;
                    if (STORE_V && a.v_out && whole) {     // the tile's own elements (not the halo) go out once
                        const int x = x0 - H + rr;
                        if (rr >= H && rr < H + kTileRows && x < R && ym < C)
                            store_streaming(a.v_out + L.elem_off + static_cast<size_t>(x) * C + ym, v);
                    }
                }
            }
            if (halo_thread) tile[hrow * PITCH + (hc < H ? PADL - 1 - hc : PADL + kTileCols + (hc - H))] = rh + gh;
        } else {
            if (FEED) feed.stash(feed_slot);
            for (int s = tid; s < ROWS * PITCH; s += 256) {
                const int rr = s / PITCH, j = s - rr * PITCH;
                const int x = x0 - H + rr, y = y0 - PADL + j;
                float v = 0.f;
                if (x >= 0 && x < R && y >= 0 && y < C) {
                    const size_t off = static_cast<size_t>(x) * C + y;
                    const bool own = rr >= H && rr < H + kTileRows && j >= PADL && j < PADL + kTileCols;
                    float gu = g[off];
                    if (MOM) {
                        gu = __fmul_rn(a.m, a.mom[L.elem_off + off]) + gu;
                        if (STORE_V && a.mom_out && whole && own) a.mom_out[L.elem_off + off] = gu;
                    }
                    v = (r ? r[off] : 0.f) + gu;
                    if (STORE_V && a.v_out && whole && own) a.v_out[L.elem_off + off] = v;
                }
                tile[s] = v;
            }
        }
        __syncthreads();

        // ---- window statistics
        // (the column as the compiler cannot see through it: otherwise it forms the 16 queue
        // entries of the thread once, outside the loop over the tiles, and keeps them in registers)
        int c0q = c0;
        asm volatile("" : "+v"(c0q));
        if (CAPTURE) {
            // Only the centres that reach the bound are wanted, and about 99.5 % do not.  A test
            // without the square root rules those out:
            //   NSI >= B  <=>  cb*sqrt(d) >= B - ca*sa  <=>  rest <= 0  or  cb^2 * d >= rest^2
            // in float32, with the slacks of PreF32 (a window whose variance cancels is never ruled out
            // on a value that is too small).  Each thread walks down its column keeping the last P row
            // sums.  The few centres that remain are queued and evaluated in full after the sweep, one
            // per thread.
            const float nf = static_cast<float>(P * P);
            float fs_a[P], fs_s[P], fs_q[P];
#pragma unroll
            for (int i = 0; i < RPT + 2 * H; ++i) {
                const float *row = &tile[(row_base + i) * PITCH + PADL + c0 - H];
                {
                    float sa = fabsf(row[0]), ss = row[0], sq = row[0] * row[0];
#pragma unroll
                    for (int j = 1; j < P; ++j) {
                        sa += fabsf(row[j]);
                        ss += row[j];
                        sq = fmaf(row[j], row[j], sq);
                    }
                    fs_a[i % P] = sa;
                    fs_s[i % P] = ss;
                    fs_q[i % P] = sq;
                }
                if (i >= 2 * H) {
                    const int o = i - 2 * H;
                    float sa = fs_a[o % P], ss = fs_s[o % P], sq = fs_q[o % P];
#pragma unroll
                    for (int j = 1; j < P; ++j) {
                        sa += fs_a[(o + j) % P];
                        ss += fs_s[(o + j) % P];
                        sq += fs_q[(o + j) % P];
                    }
                    const float nsq = nf * sq;
                    const float d_hi = fmaf(PreF32<P>::kSlack, nsq, fmaf(-ss, ss, nsq));
                    const float rest = fmaf(-caf, sa, bound_lof);
                    const int x = x0 + row_base + o, y = y0 + c0;
                    if ((rest <= 0.f || !(cb2f * d_hi < rest * rest * (1.f - 1e-6f))) && x < R && y < C) {
                        const uint32_t pos = atomicAdd(&nqueue, 1u);
                        if (pos < static_cast<uint32_t>(kQueueCap))
                            queue[pos] = static_cast<uint16_t>((row_base + o) * kTileCols + c0q);
                    }
                }
            }
        } else {
        double hs_a[P], hs_s[P], hs_q[P];
#pragma unroll
        for (int i = 0; i < RPT + 2 * H; ++i) {
            const float *row = &tile[(row_base + i) * PITCH + PADL + c0 - H];
            double w[P];
#pragma unroll
            for (int j = 0; j < P; ++j) w[j] = static_cast<double>(row[j]);
            {
                double sa = fabs(w[0]), ss = w[0], sq = w[0] * w[0];
#pragma unroll
                for (int j = 1; j < P; ++j) {
                    sa += fabs(w[j]);
                    ss += w[j];
                    sq = fma(w[j], w[j], sq);
                }
                hs_a[i % P] = sa;
                hs_s[i % P] = ss;
                hs_q[i % P] = sq;
            }
            if (i >= 2 * H) {
                const int o = i - 2 * H;   // output row inside the thread's strip
                double sa = hs_a[o % P], ss = hs_s[o % P], sq = hs_q[o % P];
#pragma unroll
                for (int j = 1; j < P; ++j) {
                    sa += hs_a[(o + j) % P];
                    ss += hs_s[(o + j) % P];
                    sq += hs_q[(o + j) % P];
                }
                const double nsq = __dmul_rn(n, sq);
                double d = var_n2_one_pass(ss, nsq);
                const int x = x0 + row_base + o, y = y0 + c0;
                {
                    // the one-pass variance cancelled (rare; never for P = 1, where it is 0 by definition)
                    if (P > 1 && d < kCancelFrac * nsq)
                        d = __dmul_rn(n, window_ssd<P>(&tile[(row_base + o) * PITCH + PADL + c0 - H], PITCH, ss / n));
                    const float out = static_cast<float>(nsi_from_var(sa, d, ca, cb));
                    if (x < R && y < C) {
                        if (MAP || (PASS == kPassSample && whole))
                            a.nsi_out[static_cast<size_t>(L.elem_off) + static_cast<size_t>(x) * C + y] = out;
                        if (FULLHIST) atomicAdd(&lhist[(__float_as_uint(out) & 0x7fffffffu) >> kCoarseShift], 1u);
                    }
                }
            }
        }
        }
        __syncthreads();                  // the sweep is complete (the tile is still needed by the queue)

        if (CAPTURE) {
            // ---- the queued centres in full: the same sums in the same order as above, Eq. 10 again
            // from the tile where the one-pass variance cancels, score, and the record if it reaches
            // the bound
            const uint32_t nq = nqueue;
            if (nq > static_cast<uint32_t>(kQueueCap) && tid == 0) a.state_rw[l].overflow = 1u;   // (more than any slot holds)
            for (uint32_t qi = tid; qi < min(nq, static_cast<uint32_t>(kQueueCap)); qi += 256) {
                const int pos = queue[qi];
                const int orow = pos / kTileCols, ocol = pos - orow * kTileCols;
                const float *win = &tile[orow * PITCH + PADL + ocol - H];
                double sa = 0.0, ss = 0.0, sq = 0.0;
#pragma unroll 1
                for (int dx = 0; dx < P; ++dx) {       // (cold code: kept rolled, it needs few registers that way)
                    const double w0 = static_cast<double>(win[dx * PITCH]);
                    double ra = fabs(w0), rs = w0, rq = w0 * w0;
#pragma unroll
                    for (int j = 1; j < P; ++j) {
                        const double wj = static_cast<double>(win[dx * PITCH + j]);
                        ra += fabs(wj);
                        rs += wj;
                        rq = fma(wj, wj, rq);
                    }
                    if (dx == 0) { sa = ra; ss = rs; sq = rq; }
                    else { sa += ra; ss += rs; sq += rq; }
                }
                const double nsq = __dmul_rn(n, sq);
                double d = var_n2_one_pass(ss, nsq);
                if (P > 1 && d < kCancelFrac * nsq) d = __dmul_rn(n, window_ssd<P>(win, PITCH, ss / n));
                const uint32_t key = __float_as_uint(static_cast<float>(nsi_from_var(sa, d, ca, cb))) & 0x7fffffffu;
                if (key >= hint_key) {
                    const uint32_t x = static_cast<uint32_t>(x0 + orow), y = static_cast<uint32_t>(y0 + ocol);
                    const uint32_t cp = atomicAdd(&ncand, 1u);
                    if (cp < static_cast<uint32_t>(kSlotCapMax)) cand[cp] = composite_key(key, x * L.C + y);
                    // fine bins upwards from the bound; the last one is open-ended
                    const uint32_t rel = (key - hint_key) >> kFineShift;
                    atomicAdd(&lhist[min(rel, static_cast<uint32_t>(kFineBins - 1))], 1u);
                }
            }
            __syncthreads();              // all reads of the tile are complete, all records made
        }

        if (CAPTURE) {
            const uint32_t nc = ncand, cap = L.slot_cap;
            unsigned long long *__restrict__ dst = a.slot_ent + L.slot_off + static_cast<size_t>(local) * cap;
            for (uint32_t i = tid; i < min(nc, cap); i += 256) dst[i] = cand[i];
            if (tid == 0) {
                a.slot_cnt[L.tile_begin_all + local] = min(nc, cap);
                if (nc > cap) a.state_rw[l].overflow = 1u;
            }
            __syncthreads();
            if (tid == 0) { ncand = 0; nqueue = 0; }
            // the next tile's first barrier orders this reset before any new append
        }
    }

    if (NBINS > 1 && cur_l != 0xffffffffu && active) {
        uint32_t *__restrict__ gh = hist_base + static_cast<size_t>(cur_l) * kHistBins;
        for (int b = tid; b < NBINS; b += 256) {
            const uint32_t c = lhist[b];
            if (c) atomicAdd(&gh[b], c);
        }
    }
}

// ------------------------------------------------------- ranking digits --
// The k_l-th largest composite key of a layer (Algorithm 1's ranking, Eq. 11's k_l) is found
// digit by digit, most significant first:
//   first digit   where the k_l-th score lies, from a histogram over all scores of the layer:
//                 candidate path: kFineBins bins of 2^kFineShift score-bit values each, counted
//                 upwards from the candidate bound by the main pass; full-map path: the top 12
//                 bits of the score, counted by the pass that writes the map (k_find0);
//   second digit  the next kLevel1Bits bits inside that bucket; the bucket's keys are gathered
//                 into the layer's list on the way (k_gather, many workgroups per layer);
//   the rest      remaining score bits, then -- only if equal scores straddle the k_l-th rank --
//                 the bits of ~index, so that the lower index wins: one workgroup per layer, on
//                 the gathered keys (k_finish).
struct DigitResult {
    uint32_t digit, above, count, found;
};

// Digit that holds the k_rem-th largest key of a histogram of nb <= 4096 bins (LDS or global),
// counted from the top; every thread of the workgroup (NW waves) returns the same result.
// `found` is 0 when the histogram holds fewer than k_rem keys.
template <int NW>
__device__ __forceinline__ DigitResult block_find_digit(const uint32_t *h, int nb, uint32_t k_rem,
                                                        uint32_t *wave_tot /*[NW]*/, DigitResult *res) {
    const int tid = threadIdx.x;
    const int per = nb >= 256 ? nb >> 8 : 1;    // the first 256 threads own `per` bins each, top bins first
    if (tid == 0) res->found = 0;
    const int hi = nb - tid * per;              // bins [hi - per, hi), as far as they exist
    uint32_t own = 0;
    if (tid < 256)
        for (int b = hi - 1; b >= hi - per && b >= 0; --b) own += h[b];
    const uint32_t incl = block_scan_incl_n<NW>(own, wave_tot);
    const uint32_t excl = incl - own;
    if (tid < 256 && excl < k_rem && k_rem <= incl) {
        uint32_t acc = excl;
        for (int b = hi - 1; b >= hi - per && b >= 0; --b) {
            const uint32_t c = h[b];
            if (acc + c >= k_rem) {
                res->digit = static_cast<uint32_t>(b);
                res->above = acc;
                res->count = c;
                res->found = 1;
                break;
            }
            acc += c;
        }
    }
    __syncthreads();
    const DigitResult r = *res;
    __syncthreads();
    return r;
}

// A candidate-path layer's threshold of this call, kept for the next calls' bounds.  The margin of
// those bounds follows what the forecasts miss: it decays slowly towards its initial value, and a
// threshold that ends s below this call's forecast (used for the bound or not) widens it to at
// least 1.5 s + 0.01 -- so the layer learns how much its threshold jitters from call to call
// without a bound having to fail first.
__device__ __forceinline__ void publish_threshold(PredState *__restrict__ pred, uint32_t l, uint32_t large,
                                                  uint32_t k, unsigned long long T) {
    if (pred == nullptr || large == 0u) return;
    PredState ps = pred[l];
    const uint32_t tau = static_cast<uint32_t>(T >> 32);
    const float init = margin_init_log2(k);
    float margin = fmaxf(init, (ps.margin > 0.f ? ps.margin : init) * kMarginDecay);
    if (ps.has_forecast && tau >= (1u << 23)) {
        const float shortfall = ps.forecast - __log2f(__uint_as_float(tau));
        // (a shortfall beyond the widest margin is a jump of the gradient's scale, not jitter: no
        // margin would have covered it, and none is sized by it)
        if (shortfall > 0.f && shortfall <= kMarginMaxLog2) margin = fmaxf(margin, kMarginSafety * shortfall + 0.01f);
    }
    ps.margin = fminf(margin, kMarginMaxLog2);
    ps.tau2 = ps.tau1;
    ps.tau1 = tau;
    pred[l] = ps;
}

// Small plans: whoever sets mask bits also counts them -- the kept elements per 8192-element chunk
// and per group of kChunkGroup chunks, which the emit turns into output positions -- and the
// counting pass over the finished mask (k_count, a launch of its own) is not needed.  A call on a
// small plan is a chain of launches of a few microseconds each; on a large one the extra atomics
// cost more than the launch (measured: VGG-19 +12 us, ResNet-18 -7 us), so large plans keep
// k_count and pass no counters here.  A mask word lies in one chunk: chunks are 256 words long and
// a layer starts at a word boundary.
struct CountCtx {
    uint32_t *chunk_cnt, *group_cnt;   // cleared at the start of the call; null: the plan counts with k_count instead
    size_t word0;                      // the layer's first mask word
    uint32_t chunk_begin, cgroup_begin;
};
__device__ __forceinline__ CountCtx count_ctx(const LayerDev &L, uint32_t *chunk_cnt, uint32_t *group_cnt) {
    return CountCtx{chunk_cnt, group_cnt, static_cast<size_t>(L.elem_off) >> 5, L.chunk_begin, L.cgroup_begin};
}
// n more kept elements in the layer's chunk number cl / in its chunk group number gl.  Many
// workgroups add to one group counter, so each has a cache line of its own (atomics on one line
// are served one after the other, 11 ns each).
__device__ __forceinline__ void count_add_chunk_only(const CountCtx &c, uint32_t cl, uint32_t n) {
    atomicAdd(&c.chunk_cnt[c.chunk_begin + cl], n);
}
__device__ __forceinline__ void count_add_group(const CountCtx &c, uint32_t gl, uint32_t n) {
    atomicAdd(&c.group_cnt[static_cast<size_t>(c.cgroup_begin + gl) * kGroupCntStride], n);
}
__device__ __forceinline__ void count_add_chunk(const CountCtx &c, uint32_t cl, uint32_t n) {
    count_add_chunk_only(c, cl, n);
    count_add_group(c, cl / kChunkGroup, n);
}
// The first wave of a workgroup hands over what the workgroup counted in LDS for the 64 chunks from
// cl0 on (lane = chunk): one add per chunk that got something, and one per chunk group -- 64
// consecutive chunks lie in at most two.
__device__ __forceinline__ void count_flush_wave0(const CountCtx &c, uint32_t cl0, uint32_t n) {
    const uint32_t lane = threadIdx.x & 63u;
    if (n) count_add_chunk_only(c, cl0 + lane, n);
    const uint32_t g0 = cl0 / kChunkGroup;
    const bool first = (cl0 + lane) / kChunkGroup == g0;
    uint32_t a = first ? n : 0u, b = first ? 0u : n;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        a += __shfl_xor(a, d, 64);
        b += __shfl_xor(b, d, 64);
    }
    if (lane == 0) {
        if (a) count_add_group(c, g0, a);
        if (b) count_add_group(c, g0 + 1, b);
    }
}
// ORs bits into mask word w and (COUNT) counts those that were not set before.
template <bool COUNT>
__device__ __forceinline__ void or_counted(const CountCtx &c, uint32_t *__restrict__ mask, size_t w, uint32_t bits) {
    if (!COUNT) {
        atomicOr(&mask[w], bits);
        return;
    }
    const uint32_t old = atomicOr(&mask[w], bits);
    const uint32_t n = __popc(bits & ~old);
    if (n) count_add_chunk(c, static_cast<uint32_t>((w - c.word0) >> 8), n);
}

// Set nbits (<= RSDGC_MAX_P) consecutive mask bits starting at bit position pos.
template <bool COUNT>
__device__ __forceinline__ void set_bits(const CountCtx &c, uint32_t *__restrict__ mask, size_t pos, uint32_t nbits) {
    const size_t w = pos >> 5;
    const uint32_t b = static_cast<uint32_t>(pos & 31);
    const uint32_t bits = (1u << nbits) - 1u;
    or_counted<COUNT>(c, mask, w, bits << b);
    if (b + nbits > 32) or_counted<COUNT>(c, mask, w + 1, bits >> (32 - b));
}

// A selected centre (flat index i inside its layer) ORs the bits of its p x p window into the
// (cleared) mask -- Section III-C: whole neighbourhoods are kept -- and its own bit into the
// centre mask when centre lists are wanted.  The words touched by different centres are nearly
// all distinct, which is the case global atomics handle well.
struct WindowGeom {
    size_t elem_off;
    int R, C, h;
};
template <bool COUNT>
__device__ __forceinline__ void mark_window(const WindowGeom &g, const CountCtx &c, uint32_t i,
                                            uint32_t *__restrict__ mask, uint32_t *__restrict__ cmask) {
    const int xc = static_cast<int>(i / static_cast<uint32_t>(g.C));
    const int yc = static_cast<int>(i - static_cast<uint32_t>(xc) * static_cast<uint32_t>(g.C));
    const int ylo = max(0, yc - g.h), yhi = min(g.C - 1, yc + g.h);
    for (int x = max(0, xc - g.h); x <= min(g.R - 1, xc + g.h); ++x)
        set_bits<COUNT>(c, mask, g.elem_off + static_cast<size_t>(x) * g.C + ylo, static_cast<uint32_t>(yhi - ylo + 1));
    if (cmask) {
        const size_t pos = g.elem_off + i;
        atomicOr(&cmask[pos >> 5], 1u << (pos & 31));
    }
}

// ----------------------------------------------------------------- hint --
// First calls with a workspace only: one workgroup per large layer that has no predicted bound
// turns the layer's sampled scores (12-bit histogram) into its candidate bound: the lower edge
// of the bucket at which the target count is reached from the top.  A layer whose sample gives
// none (too few scores, or the target only in bucket 0) goes to the full map.
__global__ __launch_bounds__(256) void k_hint(const LayerDev *__restrict__ layers,
                                              SelState *__restrict__ state,
                                              const uint32_t *__restrict__ hist_s,
                                              uint32_t *__restrict__ flags) {
    __shared__ uint32_t wave_tot[4];
    __shared__ DigitResult res;
    const int l = blockIdx.x, tid = threadIdx.x;
    const SelState st = state[l];
    const uint32_t target = layers[l].hint_target;
    constexpr int per = kHistBins / 256;
    const uint32_t *__restrict__ hs = hist_s + static_cast<size_t>(l) * kHistBins;
    const int hi = kHistBins - tid * per;          // thread 0 holds the top buckets
    uint32_t v[per];
    uint32_t own = 0;
#pragma unroll
    for (int j = 0; j < per; ++j) {                // (independent loads: one round trip)
        v[j] = hs[hi - 1 - j];
        own += v[j];
    }
    if (st.mode != kModeCandidates || st.hint_key != 0u) return;    // uniform
    if (tid == 0) res.found = 0;
    const uint32_t incl = block_scan_incl(own, wave_tot);
    const uint32_t excl = incl - own;
    if (excl < target && target <= incl) {
        uint32_t acc = excl;
#pragma unroll
        for (int j = 0; j < per; ++j) {
            if (acc < target && acc + v[j] >= target) {
                res.digit = static_cast<uint32_t>(hi - 1 - j);
                res.found = 1;
            }
            acc += v[j];
        }
    }
    __syncthreads();
    if (tid == 0) {
        const uint32_t key = res.found ? res.digit << kCoarseShift : 0u;
        if (key >= kPreF32MinKey && key <= kPreF32MaxKey) {      // (a bound the main pass can test in float32)
            state[l].hint_key = key;
        } else {
            state[l].mode = kModeFullMap;
            flags[0] = 1u;                 // the fallback pass has work
        }
    }
}

// ---------------------------------------------------------------- find0 --
// One workgroup per layer, after the NSI passes: the first ranking digit.  For a layer on the
// candidate path this is also the check of its bound: the recorded centres are usable only if
// no tile slot overflowed, at least k_l were recorded (then the k_l best of the layer are all
// among them) and the k_l-th does not lie in the open-ended top bin.  Otherwise the layer falls
// back to the full map in this call (a flag tells the fallback kernels that there is work), goes
// back to sampled bounds for the next few calls and widens the margin of its predictions.
__global__ __launch_bounds__(256) void k_find0(const LayerDev *__restrict__ layers,
                                               SelState *__restrict__ state,
                                               uint32_t *__restrict__ hist,
                                               uint32_t *__restrict__ flags,
                                               PredState *__restrict__ pred /* nullable */) {
    __shared__ uint32_t wave_tot[4];
    __shared__ DigitResult res;
    const int l = blockIdx.x, tid = threadIdx.x;
    // state, layer constants and counts are requested together: one round trip to memory
    // instead of three (each costs this one-workgroup-per-layer kernel about 2 us)
    const SelState st = state[l];
    const uint32_t large = layers[l].large;
    uint32_t *__restrict__ h = hist + static_cast<size_t>(l) * kHistBins;
    const bool cand = st.mode == kModeCandidates;                  // uniform
    const int nb = cand ? kFineBins : kHistBins, per = nb >> 8;
    const int hi = nb - tid * per;              // thread t owns bins [hi - per, hi): t = 0 holds the top bins
    constexpr int kMaxPer = kHistBins / 256;
    uint32_t v[kMaxPer];
    uint32_t own = 0;
#pragma unroll
    for (int j = 0; j < kMaxPer; ++j) {
        v[j] = j < per ? h[hi - 1 - j] : 0u;
        own += v[j];
    }
    if (st.done || st.mode == kModeSkip) return;
    // a large layer that is already on the full map (its sample gave no bound): its histogram
    // comes with the fallback pass, and the select pass finds its first digit
    if (st.mode == kModeFullMap && large != 0u) return;
    if (tid == 0) res.found = 0;
    const uint32_t incl = block_scan_incl(own, wave_tot);
    const uint32_t excl = incl - own;
    if (excl < st.k_rem && st.k_rem <= incl) {
        uint32_t acc = excl;
        bool hit = false;
#pragma unroll
        for (int j = 0; j < kMaxPer; ++j) {
            if (!hit && j < per && acc + v[j] >= st.k_rem) {
                res.digit = static_cast<uint32_t>(hi - 1 - j);
                res.above = acc;
                res.count = v[j];
                res.found = 1;
                hit = true;
            }
            if (!hit) acc += v[j];
        }
    }
    __syncthreads();
    const DigitResult r = res;
    if (cand && (!r.found || st.overflow != 0u || r.digit == static_cast<uint32_t>(kFineBins - 1) ||
                 st.hint_key == 0u)) {
        for (int b = tid; b < kFineBins; b += 256) h[b] = 0;       // the fallback pass counts afresh
        if (tid == 0) {
            SelState ns = st;
            ns.mode = kModeFullMap;
            state[l] = ns;
            flags[0] = 1u;                 // the fallback pass has work
            PredState ps = pred[l];
            ps.cooldown = kCooldownCalls;
            if (st.predicted) {
                // the margin of the predicted bounds follows the way this one failed: too few centres above
                // it -- twice the margin; a tile with too many, or a threshold beyond the bins -- the bound
                // lay too low, and a wider margin would only repeat that: half of it, down to its start value
                const float init = margin_init_log2(layers[l].k);
                const float m = ps.margin > 0.f ? ps.margin : init;
                const bool too_low = st.overflow != 0u || (r.found && r.digit == static_cast<uint32_t>(kFineBins - 1));
                ps.margin = too_low ? fmaxf(0.5f * m, init) : fminf(2.f * m, kMarginMaxLog2);
            }
            pred[l] = ps;
        }
        return;
    }
    if (tid == 0) {
        SelState ns = st;
        if (!r.found) {                    // fewer keys than k_l (cannot happen for finite input)
            ns.done = 1;
        } else {
            const uint32_t shift = cand ? kFineShift : kCoarseShift;
            ns.lo = (cand ? st.hint_key : 0u) + (r.digit << shift);
            ns.span = shift;
            ns.k_rem = st.k_rem - r.above;
            ns.T = static_cast<unsigned long long>(ns.lo) << 32;
            if (r.count == ns.k_rem) {     // whole bucket taken: the threshold is its lower edge
                ns.done = 1;
                publish_threshold(pred, l, large, layers[l].k, ns.T);
            }
        }
        state[l] = ns;
    }
}

// --------------------------------------------------------------- gather --
// After the first digit: the keys of each layer's threshold bucket (score bits in
// [lo, lo + 2^span)) are copied into the layer's list and their next digit is histogrammed.
// Three kinds of workgroups share the launch:
//   [0, n_map_wgs)              stride over the plan's list of 8192-element score-map chunks
//                               (layers that are always ranked on the full map);
//   [n_map_wgs, +n_slot_wgs)    stride over the plan's list of slot groups (large layers,
//                               where they are still in candidate mode);
//   the last n_fb_wgs           only when some large layer fell back to the full map: they
//                               walk all chunks and take those of such layers (and find the
//                               first digit of such a layer themselves, from the histogram the
//                               fallback pass has counted).
// Matches from the score map are staged in LDS and appended with one atomic per flush.
// The recorded candidates of a large layer are nearly all decided by the first digit already
// (its bins are fine: the threshold bucket holds a per cent or two of them): a candidate above
// the bucket is selected whatever the later digits say, so its window is marked here and now
// (k_mark marks the few that the bucket contributes); one in the bucket is appended to the
// list straight away, one atomic per wave, without staging or barriers.
// (In-kernel hand-over of a finished layer to "the last workgroup" was measured and dropped:
// the device-scope fences it needs write back the whole L2 of an XCD each time and cost more
// than the launch they save.)
constexpr int kStage = 2048;            // staged keys per workgroup (a round adds at most 1024)
constexpr int kSlotsPerWave = kSlotGroup / 4;   // tile slots of a group that one wave of a gather workgroup takes

constexpr int kTileMaskWords = kTileRows * kTileCols / 32;    // mask words of one tile (rows of 8 words)
constexpr int kGatherCountSlots = 64;                          // chunks a group of tiles counts for in LDS (the rest: directly)

struct GatherShared {
    union {
        unsigned long long ent[kStage];               // score-map roles: staged keys
        struct {                                      // slot role:
            uint32_t bits[kSlotGroup * kTileMaskWords];   // mask words of the group of tiles being written
            uint32_t ccnt[kGatherCountSlots];             // bits set, per chunk from the group's first one on
        };
    };
    uint32_t hist[kLevel1Bins];         // second-digit counts
    DigitResult res;
    uint32_t n;                         // staged keys
    uint32_t base;
};

struct GatherLists {
    const DirEntry *chunk_dir;       // all chunks by layer (fallback walk)
    const ChunkEntry *map_chunks;    // [n_map_chunks]
    const GroupEntry *cand_groups;   // [n_cand_groups]
    uint32_t n_layers, n_chunks, n_map_chunks, n_cand_groups;
    uint32_t n_map_wgs, n_slot_wgs;  // the remaining workgroups are fallback walkers
};

struct GatherArgs {
    const LayerDev *layers;
    const SelState *state;
    const uint32_t *keys;                 // score map
    const uint32_t *slot_cnt;
    const unsigned long long *slot_ent;
    uint32_t *list_cnt;
    unsigned long long *list_ent;
    const uint32_t *hist;                 // first-digit counts (fallback layers)
    uint32_t *hist1;                      // [n_layers][kLevel1Bins]
    const uint32_t *flags;
    uint32_t *mask, *cmask;               // kept-element bitmask; selected-centre bitmask (nullable)
    uint32_t *chunk_cnt, *group_cnt;      // kept elements per chunk / chunk group, counted as the bits are set
};

// The list of the layer the workgroup is working on.
struct GatherList {
    uint32_t *cnt;                        // this workgroup's shard counter
    unsigned long long *ent;              // ... and region
    uint32_t cap;
};

// Appends the staged keys to the current layer's list.
__device__ __forceinline__ void gather_flush_keys(GatherShared &sh, const GatherList &gl) {
    __syncthreads();
    const uint32_t n = sh.n;
    if (n != 0) {                          // uniform
        if (threadIdx.x == 0) sh.base = atomicAdd(gl.cnt, n);
        __syncthreads();
        const uint32_t base = sh.base;
        for (uint32_t i = threadIdx.x; i < n; i += 256)
            if (base + i < gl.cap) gl.ent[base + i] = sh.ent[i];
        __syncthreads();
        if (threadIdx.x == 0) sh.n = 0;
    }
    __syncthreads();
}

// One round of at most 1024 appends (4 per thread) is about to start: make room for it.
__device__ __forceinline__ void gather_make_room(GatherShared &sh, const GatherList &gl) {
    __syncthreads();                       // appends of the previous round are counted
    if (sh.n + 1024u > static_cast<uint32_t>(kStage))            // uniform
        gather_flush_keys(sh, gl);
}

// Stages key K (of a flagged lane) and counts its second digit.  Called by whole waves.
__device__ __forceinline__ void gather_stage_key(GatherShared &sh, bool hit, unsigned long long K,
                                                 uint32_t lo, uint32_t shift1) {
    const uint32_t pos = wave_append(&sh.n, hit);
    if (hit) {
        sh.ent[pos] = K;
        atomicAdd(&sh.hist[(static_cast<uint32_t>(K >> 32) - lo) >> shift1], 1u);
    }
}

template <bool COUNT>
__global__ __launch_bounds__(256) void k_gather(const GatherArgs a, const GatherLists gl) {
    __shared__ GatherShared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // role 0: listed score-map chunks, 1: listed slot groups, 2: fallback walk over all chunks
    const int role = blockIdx.x < gl.n_map_wgs ? 0 : blockIdx.x < gl.n_map_wgs + gl.n_slot_wgs ? 1 : 2;
    const uint32_t first = role == 0 ? blockIdx.x : role == 1 ? blockIdx.x - gl.n_map_wgs
                                                              : blockIdx.x - gl.n_map_wgs - gl.n_slot_wgs;
    const uint32_t stride = role == 0 ? gl.n_map_wgs : role == 1 ? gl.n_slot_wgs
                                                                 : gridDim.x - gl.n_map_wgs - gl.n_slot_wgs;
    const uint32_t n_items = role == 0 ? gl.n_map_chunks : role == 1 ? gl.n_cand_groups : gl.n_chunks;
    const DirEntry *__restrict__ dir = gl.chunk_dir;
    if (first >= n_items) return;
    if (role == 2 && a.flags[0] == 0u) return;
    if (tid == 0) sh.n = 0;
    for (int b = tid; b < kLevel1Bins; b += 256) sh.hist[b] = 0;
    __syncthreads();

    uint32_t e = role == 2 ? dir_lookup(dir, gl.n_layers, first) : 0u;
    uint32_t cur_l = 0xffffffffu;
    bool active = false;
    uint32_t lo = 0, width = 0, shift1 = 0;   // the current layer's bucket [lo, lo + width) and its second digit's shift
    uint32_t above = 0;                       // candidate layers: scores from here on are selected for certain
    LayerDev L;
    GatherList list = {nullptr, nullptr, 0u};

    for (uint32_t it = first; it < n_items; it += stride) {
        uint32_t l;
        ChunkEntry ce = {};
        GroupEntry ge = {};
        if (role == 0) {
            ce = gl.map_chunks[it];
            l = ce.layer;
        } else if (role == 1) {
            ge = gl.cand_groups[it];
            l = ge.layer;
        } else {
            e = dir_advance(dir, gl.n_layers, e, it);
            l = dir[e].layer;
        }
        if (l != cur_l) {
            if (active) {                  // uniform: the finished layer's keys and counts go out
                gather_flush_keys(sh, list);
                uint32_t *__restrict__ gh = a.hist1 + static_cast<size_t>(cur_l) * kLevel1Bins;
                for (int b = tid; b < kLevel1Bins; b += 256) {
                    const uint32_t cc = sh.hist[b];
                    if (cc) { atomicAdd(&gh[b], cc); sh.hist[b] = 0; }
                }
                __syncthreads();
            }
            cur_l = l;
            L = a.layers[l];
            const SelState st = a.state[l];
            active = !st.done && st.mode == (role == 1 ? kModeCandidates : kModeFullMap);
            lo = st.lo;
            width = 1u << st.span;
            shift1 = st.span - kLevel1Bits;
            if (role == 1) {
                // candidates: everything at or above `above` is selected for certain.  A layer whose
                // first digit already settled the ranking (done) has its threshold at lo.
                active = st.mode == kModeCandidates;
                above = st.done ? static_cast<uint32_t>(st.T >> 32) : lo + width;
                if (st.done) width = 0;
            }
            if (role == 2) {
                active = st.mode == kModeFullMap && L.large != 0u;      // the others are on the list
                if (active) {              // uniform: first digit from the histogram of the fallback pass
                    if (tid < 64) {
                        const WaveBucket wb = wave_find_bucket(a.hist + static_cast<size_t>(l) * kHistBins, L.k);
                        if (tid == 0) sh.res = DigitResult{wb.bucket, wb.above, wb.count, wb.found};
                    }
                    __syncthreads();
                    const DigitResult r = sh.res;
                    __syncthreads();
                    lo = r.found ? r.digit << kCoarseShift : 0u;
                    width = 1u << kCoarseShift;
                    shift1 = kCoarseShift - kLevel1Bits;
                    if (!r.found || r.count == L.k - r.above) active = false;   // nothing left to rank
                }
            }
            // the workgroup's shard of the layer's list: its own counter (own cache line) and region
            const uint32_t shard = blockIdx.x % L.list_shards;
            list.cap = L.list_cap / L.list_shards;
            list.cnt = a.list_cnt + (static_cast<size_t>(l) * kListShards + shard) * kListCntStride;
            list.ent = a.list_ent + L.list_off + static_cast<size_t>(shard) * list.cap;
        }
        if (!active) {
            if (role == 2) {               // on to this workgroup's first chunk of the next layer
                const uint32_t nb = dir[e + 1].begin;
                it += (nb - it + stride - 1) / stride * stride - stride;
            }
            continue;
        }
        if (role != 1) {
            if (role == 2) {
                ce.start = (it - L.chunk_begin) * kChunk;
                ce.len = min(static_cast<uint32_t>(kChunk), L.G - ce.start);
                ce.arena_off = static_cast<uint64_t>(L.elem_off) + ce.start;
            }
            const uint32_t start = ce.start, len = ce.len;
            const uint32_t *__restrict__ src = a.keys + ce.arena_off;
            // half a chunk is requested before any of it is used
            constexpr int NQ = kChunk / 2048;
#pragma unroll 1
            for (uint32_t half = 0; half < 2u && half * (kChunk / 2) < len; ++half) {
                uint4 q[NQ];
#pragma unroll
                for (int j = 0; j < NQ; ++j) {
                    const uint32_t e4 = half * (kChunk / 2) + j * 1024 + 4 * tid;
                    q[j] = make_uint4(0, 0, 0, 0);
                    if (e4 + 3 < len) {
                        q[j] = *reinterpret_cast<const uint4 *>(src + e4);
                    } else if (e4 < len) {
                        q[j].x = src[e4];
                        if (e4 + 1 < len) q[j].y = src[e4 + 1];
                        if (e4 + 2 < len) q[j].z = src[e4 + 2];
                    }
                }
#pragma unroll
                for (int j = 0; j < NQ; ++j) {
                    const uint32_t e4 = half * (kChunk / 2) + j * 1024 + 4 * tid;
                    if (half * (kChunk / 2) + static_cast<uint32_t>(j) * 1024u >= len) break;       // uniform
                    gather_make_room(sh, list);
                    const uint32_t kk[4] = {q[j].x, q[j].y, q[j].z, q[j].w};
#pragma unroll
                    for (uint32_t c = 0; c < 4; ++c) {
                        const bool hit = e4 + c < len && (kk[c] & 0x7fffffffu) - lo < width;
                        gather_stage_key(sh, hit, composite_key(kk[c], start + e4 + c), lo, shift1);
                    }
                }
            }
        } else {
            const uint32_t slot_cap = L.slot_cap;
            const unsigned long long *__restrict__ ent0 =
                a.slot_ent + L.slot_off + static_cast<size_t>(ge.slot0 - L.tile_begin_all) * slot_cap;
            const WindowGeom geom = {static_cast<size_t>(L.elem_off), static_cast<int>(L.R), static_cast<int>(L.C),
                                     (static_cast<int>(L.p) - 1) / 2};
            const CountCtx cctx = count_ctx(L, a.chunk_cnt, a.group_cnt);
            if ((L.C & 31u) == 0u) {
                // Rows of whole mask words: every mask word of the layer lies in exactly one tile.  The
                // workgroup builds the words of its group of tiles in LDS from the group's own candidates
                // and writes them with plain stores, whole cache lines at a time -- except the words that
                // windows of other groups' candidates can reach (the h rows along a tile's upper and lower
                // edge, the first and last word of the group's run of tiles): those, and the bits that the
                // group's windows set in other groups' tiles, are ORed into the (cleared) mask.
                // The bits are counted as they are set (an OR tells which were new), per chunk, in LDS
                // first: a group of tiles lies in a few chunks.
                const int h = geom.h, C = geom.C, R = geom.R;
                const int tiles_x = static_cast<int>(L.tiles_x);
                const int g0 = static_cast<int>(ge.slot0 - L.tile_begin_all), gn = static_cast<int>(ge.ntile);
                // first chunk that the group's windows can reach: that of the element h rows above and h
                // columns left of the first tile's corner
                const uint32_t cl0 = static_cast<uint32_t>(
                    (static_cast<size_t>(max(0, (g0 / tiles_x) * kTileRows - h)) * C +
                     static_cast<size_t>(max(0, (g0 % tiles_x) * kTileCols - h))) / kChunk);
                __syncthreads();                                 // (the previous group's words are written)
                for (int i = tid; i < kSlotGroup * kTileMaskWords; i += 256) sh.bits[i] = 0u;
                if (COUNT && tid < kGatherCountSlots) sh.ccnt[tid] = 0u;
                __syncthreads();
                {
                    // sixteen lanes per tile slot; a round covers 16 entries of each
                    const int sidx0 = tid >> 4;
                    const uint32_t cnt = sidx0 < gn ? min(a.slot_cnt[ge.slot0 + static_cast<uint32_t>(sidx0)], slot_cap) : 0u;
                    for (uint32_t j = static_cast<uint32_t>(tid) & 15u; j < cnt; j += 16u) {
                        const unsigned long long K = ent0[static_cast<size_t>(sidx0) * slot_cap + j];
                        const uint32_t score = static_cast<uint32_t>(K >> 32);
                        if (score >= above) {                    // selected for certain: its window, tile by tile
                            const uint32_t i = ~static_cast<uint32_t>(K);
                            const int xc = static_cast<int>(i / static_cast<uint32_t>(C));
                            const int yc = static_cast<int>(i - static_cast<uint32_t>(xc) * static_cast<uint32_t>(C));
                            const int wx0 = max(0, xc - h), wx1 = min(R - 1, xc + h);
                            const int wy0 = max(0, yc - h), wy1 = min(C - 1, yc + h);
                            for (int tr = wx0 / kTileRows; tr <= wx1 / kTileRows; ++tr)
                                for (int tc = wy0 / kTileCols; tc <= wy1 / kTileCols; ++tc) {
                                    const int sidx = tr * tiles_x + tc - g0;
                                    const bool mine = static_cast<uint32_t>(sidx) < static_cast<uint32_t>(gn);
                                    const int r0 = tr * kTileRows, c0 = tc * kTileCols;
                                    const int xa = max(r0, wx0), xb = min(r0 + kTileRows - 1, wx1);
                                    const int ya = max(c0, wy0) - c0, yb = min(c0 + kTileCols - 1, wy1) - c0;
                                    const uint32_t w0 = static_cast<uint32_t>(ya) >> 5, b0 = static_cast<uint32_t>(ya) & 31u;
                                    const uint32_t len = static_cast<uint32_t>(yb - ya + 1);
                                    const uint32_t run = (1u << len) - 1u;
                                    for (int x = xa; x <= xb; ++x) {
                                        if (mine) {
                                            uint32_t *row = sh.bits + sidx * kTileMaskWords + (x - r0) * (kTileCols / 32);
                                            atomicOr(&row[w0], run << b0);
                                            if (b0 + len > 32u) atomicOr(&row[w0 + 1], run >> (32u - b0));
                                        } else if (!COUNT) { // another group's tile: straight into the mask
                                            uint32_t *row = a.mask + ((geom.elem_off + static_cast<size_t>(x) * C + c0) >> 5);
                                            atomicOr(&row[w0], run << b0);
                                            if (b0 + len > 32u) atomicOr(&row[w0 + 1], run >> (32u - b0));
                                        } else {             // ... and the new bits counted
                                            const size_t wrow = (static_cast<size_t>(x) * C + c0) >> 5;   // first word of the tile row, inside the layer
                                            uint32_t *row = a.mask + (geom.elem_off >> 5) + wrow;
#pragma unroll
                                            for (uint32_t part = 0; part < 2u; ++part) {
                                                const uint32_t bits = part == 0u ? run << b0 : (b0 + len > 32u ? run >> (32u - b0) : 0u);
                                                if (bits == 0u) continue;
                                                const uint32_t fresh = __popc(bits & ~atomicOr(&row[w0 + part], bits));
                                                if (fresh) {
                                                    const uint32_t slot = static_cast<uint32_t>((wrow + w0 + part) >> 8) - cl0;
                                                    if (slot < static_cast<uint32_t>(kGatherCountSlots)) atomicAdd(&sh.ccnt[slot], fresh);
                                                    else count_add_chunk(cctx, cl0 + slot, fresh);
                                                }
                                            }
                                        }
                                    }
                                }
                            if (a.cmask) {
                                const size_t pos = geom.elem_off + i;
                                atomicOr(&a.cmask[pos >> 5], 1u << (pos & 31));
                            }
                        } else if (score - lo < width) {         // in the threshold bucket (never when the layer is done):
                            const uint32_t pos = atomicAdd(list.cnt, 1u);       // few of them, one atomic each
                            if (pos < list.cap) list.ent[pos] = K;
                            atomicAdd(&sh.hist[(score - lo) >> shift1], 1u);
                        }
                    }
                }
                __syncthreads();
                // The group's words.  Neighbouring tiles of one tile row are neighbours in memory:
                // consecutive threads walk along a matrix row through the group's tiles, so a wave writes
                // whole cache lines.  Words past the end of a matrix row or below the last row do not exist.
                for (int i = tid; i < gn * kTileMaskWords; i += 256) {
                    const int rr = i / (gn * 8), rem = i - rr * (gn * 8), sidx = rem >> 3, ww = rem & 7;
                    const int local = g0 + sidx, tr = local / tiles_x, tc = local - tr * tiles_x;
                    const int x = tr * kTileRows + rr, y = tc * kTileCols + 32 * ww;
                    if (x < R && y < C) {
                        const uint32_t word = sh.bits[sidx * kTileMaskWords + rr * 8 + ww];
                        const size_t e0 = static_cast<size_t>(x) * C + y;
                        uint32_t *dst = a.mask + ((geom.elem_off + e0) >> 5);
                        const bool shared = (rr < h && tr > 0) || (rr >= kTileRows - h && x + h >= (tr + 1) * kTileRows && (tr + 1) * kTileRows < R) ||
                                            (ww == 0 && sidx == 0 && tc > 0) ||
                                            (ww == 7 && sidx == gn - 1 && tc < tiles_x - 1);
                        uint32_t fresh = word;
                        if (!shared) *dst = word;
                        else if (word != 0u) {
                            if (COUNT) fresh = word & ~atomicOr(dst, word);
                            else atomicOr(dst, word);
                        }
                        if (COUNT && fresh) {
                            const uint32_t slot = static_cast<uint32_t>(e0 / kChunk) - cl0;
                            if (slot < static_cast<uint32_t>(kGatherCountSlots)) atomicAdd(&sh.ccnt[slot], __popc(fresh));
                            else count_add_chunk(cctx, cl0 + slot, __popc(fresh));
                        }
                    }
                }
                static_assert(kGatherCountSlots == 64, "one lane of the first wave per counted chunk");
                if (COUNT) {
                    __syncthreads();
                    if (tid < 64) count_flush_wave0(cctx, cl0, sh.ccnt[tid]);
                }
            } else {
            // each wave takes 4 of the group's tile slots; a round covers 64 entries of each
            uint32_t cnt[kSlotsPerWave];
            uint32_t longest = 0;
#pragma unroll
            for (int c = 0; c < kSlotsPerWave; ++c) {
                const uint32_t s = static_cast<uint32_t>(wave) + 4u * c;
                cnt[c] = s < ge.ntile ? min(a.slot_cnt[ge.slot0 + s], slot_cap) : 0u;
                longest = max(longest, cnt[c]);                     // wave-uniform
            }
            for (uint32_t j0 = 0; j0 < longest; j0 += 64) {
                const uint32_t j = j0 + lane;
                unsigned long long K[kSlotsPerWave];
#pragma unroll
                for (int c = 0; c < kSlotsPerWave; ++c)
                    K[c] = j < cnt[c] ? ent0[static_cast<size_t>(wave + 4 * c) * slot_cap + j] : 0ull;
#pragma unroll
                for (int c = 0; c < kSlotsPerWave; ++c) {
                    const uint32_t score = static_cast<uint32_t>(K[c] >> 32);
                    const bool valid = j < cnt[c];
                    if (valid && score >= above) mark_window<COUNT>(geom, cctx, ~static_cast<uint32_t>(K[c]), a.mask, a.cmask);
                    const bool hit = valid && score < above && score - lo < width;    // (never when the layer is done)
                    const unsigned long long m = __ballot(hit);
                    if (m != 0ull) {       // wave-uniform
                        const uint32_t leader = static_cast<uint32_t>(__ffsll(static_cast<long long>(m))) - 1u;
                        uint32_t base = 0;
                        if (static_cast<uint32_t>(lane) == leader) base = atomicAdd(list.cnt, static_cast<uint32_t>(__popcll(m)));
                        base = __shfl(base, static_cast<int>(leader), 64);
                        if (hit) {
                            const uint32_t pos = base + static_cast<uint32_t>(__popcll(m & ((1ull << lane) - 1ull)));
                            if (pos < list.cap) list.ent[pos] = K[c];
                            atomicAdd(&sh.hist[(score - lo) >> shift1], 1u);
                        }
                    }
                }
            }
            }
        }
    }
    if (active) {
        gather_flush_keys(sh, list);
        uint32_t *__restrict__ gh = a.hist1 + static_cast<size_t>(cur_l) * kLevel1Bins;
        for (int b = tid; b < kLevel1Bins; b += 256) {
            const uint32_t cc = sh.hist[b];
            if (cc) atomicAdd(&gh[b], cc);
        }
    }
}

// --------------------------------------------------------------- filter --
// Only for plans with large layers that are ranked on the full map (a block grid, a keep ratio
// too high for the candidate path): the threshold bucket of such a layer holds hundreds of
// thousands of keys, too many for the one workgroup of k_finish to go through.  kFilterSplit
// workgroups per layer find the second digit (each for itself, from the layer's complete
// histogram) and copy the keys of the list that share it -- a few hundred -- to the layer's
// second, small list, from which k_finish then works.
constexpr int kFilterSplit = 32;
constexpr int kFilterThreads = 1024;
constexpr int kList2Cap = 2048;          // == kStage: what k_finish can hold in LDS

__global__ __launch_bounds__(kFilterThreads) void k_filter(const LayerDev *__restrict__ layers,
                                                           const SelState *__restrict__ state,
                                                           const uint32_t *__restrict__ hist1,
                                                           const uint32_t *__restrict__ list_cnt,
                                                           const unsigned long long *__restrict__ list_ent,
                                                           uint32_t *__restrict__ list2_cnt,
                                                           unsigned long long *__restrict__ list2_ent) {
    __shared__ uint32_t lh[kLevel1Bins];
    __shared__ unsigned long long stage[kList2Cap];
    __shared__ uint32_t wave_tot[kFilterThreads / 64];
    __shared__ DigitResult res;
    __shared__ uint32_t nstage, base_pos;
    const int l = blockIdx.x / kFilterSplit, part = blockIdx.x % kFilterSplit, tid = threadIdx.x;
    // lane s of every wave reads shard s's counter (unused shards stay 0); issued with the other loads
    const uint32_t *__restrict__ cnt = list_cnt + static_cast<size_t>(l) * kListShards * kListCntStride;
    const uint32_t c = (tid & 63) < kListShards ? cnt[(tid & 63) * kListCntStride] : 0u;
    const SelState st = state[l];
    const LayerDev L = layers[l];
    for (int b = tid; b < kLevel1Bins; b += kFilterThreads) lh[b] = hist1[static_cast<size_t>(l) * kLevel1Bins + b];
    // (a large layer that fell back to the full map has its first digit found in the gather pass only:
    // k_finish goes through its list alone -- rare)
    if (st.done || st.mode != kModeFullMap || L.large != 0u) return;
    uint32_t total = c;
#pragma unroll
    for (int d = 8; d >= 1; d >>= 1) total += __shfl_xor(total, d, 64);
    total = __shfl(total, 0, 64);
    const uint32_t shards = L.list_shards, cap = L.list_cap / shards;
    if (total <= static_cast<uint32_t>(kList2Cap) || __syncthreads_or(c > cap)) return;   // small enough, or overflowed
    const DigitResult r = block_find_digit<kFilterThreads / 64>(lh, kLevel1Bins, st.k_rem, wave_tot, &res);
    if (!r.found || r.count == st.k_rem - r.above) return;       // nothing left to rank below this digit
    const uint32_t sh1 = st.span - kLevel1Bits;
    const unsigned long long base = (static_cast<unsigned long long>(st.lo) << 32) +
                                    (static_cast<unsigned long long>(r.digit) << (32 + sh1));
    const int top = 32 + static_cast<int>(sh1);
    // this workgroup's shard, and its share of that shard
    const uint32_t shard = part % shards, sub = part / shards, nsub = (kFilterSplit + shards - 1 - shard) / shards;
    const uint32_t n = __shfl(c, static_cast<int>(shard), 64);
    const unsigned long long *__restrict__ list = list_ent + L.list_off + static_cast<size_t>(shard) * cap;
    if (tid == 0) nstage = 0;
    __syncthreads();
    constexpr uint32_t U = 4;              // independent loads in flight per thread
    for (uint32_t i0 = sub * U * kFilterThreads; i0 < n; i0 += nsub * U * kFilterThreads) {
        unsigned long long K[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t i = i0 + u * kFilterThreads + tid;
            K[u] = i < n ? list[i] : 0ull;
        }
#pragma unroll
        for (uint32_t u = 0; u < U; ++u)
            if (i0 + u * kFilterThreads + tid < n && K[u] >= base && ((K[u] - base) >> top) == 0ull) {
                const uint32_t pos = atomicAdd(&nstage, 1u);
                if (pos < static_cast<uint32_t>(kList2Cap)) stage[pos] = K[u];
            }
    }
    __syncthreads();
    const uint32_t m = nstage;
    if (m == 0) return;                    // uniform
    if (tid == 0) base_pos = atomicAdd(&list2_cnt[l], m);        // counts past the capacity too
    __syncthreads();
    const uint32_t b0 = base_pos;
    for (uint32_t i = tid; i < min(m, static_cast<uint32_t>(kList2Cap)); i += kFilterThreads)
        if (b0 + i < static_cast<uint32_t>(kList2Cap))
            list2_ent[static_cast<size_t>(l) * kList2Cap + b0 + i] = stage[i];
}

// --------------------------------------------------------------- finish --
// One workgroup (1024 threads) per layer finishes the ranking: second digit from the layer's
// histogram; if the k-th rank is still inside a bucket of several keys, the bucket's keys are
// staged in LDS from the layer's list and the remaining score bits and -- only if equal
// scores straddle the k-th rank -- the bits of ~index are resolved there, so that the lower
// index wins.  Slow but exact routes: if the bucket's keys do not fit the stage, each further
// digit streams the list again; if the list itself overflowed (a huge number of nearly equal
// scores, e.g. an all-zero layer), each digit streams the layer's keys from the score map or
// the tile slots.
constexpr int kFinishThreads = 1024;
constexpr int kFinishWaves = kFinishThreads / 64;

// Calls f(K) for every key of a layer's list.  `c` holds, in lane s of every wave, the number of
// keys in shard s.  The shards are walked side by side -- one load per shard in flight per
// thread -- rather than one after the other: a shard of a few hundred keys is one round trip to
// memory, and sixteen of them in a row were most of this kernel's time.
template <typename F>
__device__ __forceinline__ void for_each_list_key(const unsigned long long *__restrict__ list, uint32_t shards,
                                                  uint32_t cap, uint32_t c, F f) {
    uint32_t longest = c;
#pragma unroll
    for (int d = 8; d >= 1; d >>= 1) longest = max(longest, __shfl_xor(longest, d, 64));
    longest = __shfl(longest, 0, 64);
    for (uint32_t i = threadIdx.x; i < longest + threadIdx.x; i += kFinishThreads) {   // (the same trip count in every thread)
        unsigned long long K[kListShards];
        bool have[kListShards];
#pragma unroll
        for (int s = 0; s < kListShards; ++s) {
            have[s] = static_cast<uint32_t>(s) < shards && i < __shfl(c, s, 64);
            K[s] = have[s] ? list[static_cast<size_t>(s) * cap + i] : 0ull;
        }
#pragma unroll
        for (int s = 0; s < kListShards; ++s)
            if (have[s]) f(K[s]);
    }
}

__global__ __launch_bounds__(kFinishThreads) void k_finish(const LayerDev *__restrict__ layers,
                                                           SelState *__restrict__ state,
                                                           const uint32_t *__restrict__ hist,
                                                           const uint32_t *__restrict__ hist1,
                                                           const uint32_t *__restrict__ list_cnt,
                                                           const unsigned long long *__restrict__ list_ent,
                                                           const uint32_t *__restrict__ keys,
                                                           const uint32_t *__restrict__ slot_cnt,
                                                           const unsigned long long *__restrict__ slot_ent,
                                                           const uint32_t *__restrict__ list2_cnt,
                                                           const unsigned long long *__restrict__ list2_ent,
                                                           PredState *__restrict__ pred /* nullable */) {
    __shared__ uint32_t lh[kLevel1Bins];
    __shared__ unsigned long long sel[kStage];
    __shared__ uint32_t wave_tot[kFinishWaves];
    __shared__ DigitResult res;
    __shared__ uint32_t nstage;
    const int l = blockIdx.x, tid = threadIdx.x;
    // lane s of every wave reads shard s's counter (unused shards stay 0); issued with the other loads
    const uint32_t *__restrict__ cnt = list_cnt + static_cast<size_t>(l) * kListShards * kListCntStride;
    const uint32_t c = (tid & 63) < kListShards ? cnt[(tid & 63) * kListCntStride] : 0u;
    const uint32_t n2 = list2_cnt[l];     // keys that k_filter has already picked from a long list (0: none)
    const SelState st = state[l];
    const LayerDev L = layers[l];
    for (int b = tid; b < kLevel1Bins; b += kFinishThreads) lh[b] = hist1[static_cast<size_t>(l) * kLevel1Bins + b];
    if (st.done || st.mode == kModeSkip) return;
    __syncthreads();
    uint32_t lo = st.lo, span = st.span, k_rem = st.k_rem;
    if (st.mode == kModeFullMap && L.large != 0u) {
        // a large layer that fell back to the full map: its first digit, as the gather pass found it
        __shared__ uint32_t lh0[kHistBins];
        for (int b = tid; b < kHistBins; b += kFinishThreads) lh0[b] = hist[static_cast<size_t>(l) * kHistBins + b];
        __syncthreads();
        const DigitResult r0 = block_find_digit<kFinishWaves>(lh0, kHistBins, L.k, wave_tot, &res);
        lo = r0.found ? r0.digit << kCoarseShift : 0u;
        span = kCoarseShift;
        k_rem = r0.found ? L.k - r0.above : 0u;
        if (!r0.found || r0.count == k_rem) {      // nothing left to rank
            if (tid == 0) {
                SelState ns = st;
                ns.T = static_cast<unsigned long long>(lo) << 32;
                ns.lo = lo;
                ns.span = span;
                ns.k_rem = k_rem;
                ns.done = 1;
                state[l] = ns;
                publish_threshold(pred, l, L.large, L.k, ns.T);
            }
            return;
        }
    }
    const uint32_t shards = L.list_shards, cap = L.list_cap / shards;
    const bool use_list = __syncthreads_and(c <= cap) != 0;      // every shard of the list fits
    DigitResult r = block_find_digit<kFinishWaves>(lh, kLevel1Bins, k_rem, wave_tot, &res);
    const uint32_t sh1 = span - kLevel1Bits;                     // score bits still open after this digit
    unsigned long long T = static_cast<unsigned long long>(lo) << 32;
    bool done = !r.found;                  // fewer keys than k_rem (cannot happen for finite input)
    if (r.found) {
        T += static_cast<unsigned long long>(r.digit) << (32 + sh1);
        k_rem -= r.above;
        done = r.count == k_rem;           // whole bucket taken: the threshold is its lower edge
    }
    if (!done) {
        // Keys still in question: K - T < 2^(32 + sh1).  Their remaining bits are ranked as the
        // number rel = K - T, most significant digit first.
        const unsigned long long base = T;
        const int top = 32 + static_cast<int>(sh1);
        const unsigned long long *__restrict__ list = list_ent + L.list_off;
        uint32_t nsel = 0xffffffffu;
        if (use_list && n2 != 0u && n2 <= static_cast<uint32_t>(kStage)) {   // already picked by k_filter
            for (uint32_t i = tid; i < n2; i += kFinishThreads)
                sel[i] = list2_ent[static_cast<size_t>(l) * kList2Cap + i] - base;
            __syncthreads();
            nsel = n2;
        } else if (use_list) {             // stage the bucket's keys
            if (tid == 0) nstage = 0;
            __syncthreads();
            for_each_list_key(list, shards, cap, c, [&](unsigned long long K) {
                if (K >= base && ((K - base) >> top) == 0ull) {
                    const uint32_t pos = atomicAdd(&nstage, 1u);
                    if (pos < static_cast<uint32_t>(kStage)) sel[pos] = K - base;
                }
            });
            __syncthreads();
            nsel = nstage;
        }
        const bool staged = nsel <= static_cast<uint32_t>(kStage);
        unsigned long long Trel = 0;
        int shift_prev = top;
#pragma unroll 1
        for (int lv = 0; lv < 4 && !done; ++lv) {
            const int shift = lv == 0 ? 32 : lv == 1 ? 21 : lv == 2 ? 10 : 0;
            const int nb = 1 << (shift_prev - shift);            // 2^sh1 (4 or 256), 2048, 2048, 1024
            __syncthreads();
            for (int b = tid; b < nb; b += kFinishThreads) lh[b] = 0;
            __syncthreads();
            const unsigned long long want = Trel >> shift_prev;
#define RSDGC_COUNT_KEY(K_)                                                                         \
    {                                                                                               \
        const unsigned long long k_ = (K_);                                                         \
        if (k_ >= base && ((k_ - base) >> shift_prev) == want)                                      \
            atomicAdd(&lh[static_cast<uint32_t>((k_ - base) >> shift) & (nb - 1)], 1u);             \
    }
            if (staged) {
                for (uint32_t i = tid; i < nsel; i += kFinishThreads) {
                    const unsigned long long rel = sel[i];
                    if ((rel >> shift_prev) == want) atomicAdd(&lh[static_cast<uint32_t>(rel >> shift) & (nb - 1)], 1u);
                }
            } else if (use_list) {
                for_each_list_key(list, shards, cap, c, [&](unsigned long long K) { RSDGC_COUNT_KEY(K) });
            } else if (st.mode == kModeFullMap) {
                const uint32_t *__restrict__ src = keys + L.elem_off;
                for (uint32_t i = tid; i < L.G; i += kFinishThreads) RSDGC_COUNT_KEY(composite_key(src[i], i))
            } else {
                for (uint32_t t = tid >> 8; t < L.n_tiles; t += kFinishThreads / 256) {
                    const uint32_t n = min(slot_cnt[L.tile_begin_all + t], L.slot_cap);
                    const unsigned long long *__restrict__ ent = slot_ent + L.slot_off + static_cast<size_t>(t) * L.slot_cap;
                    for (uint32_t i = tid & 255; i < n; i += 256) RSDGC_COUNT_KEY(ent[i])
                }
            }
#undef RSDGC_COUNT_KEY
            __syncthreads();
            r = block_find_digit<kFinishWaves>(lh, nb, k_rem, wave_tot, &res);
            if (!r.found) break;           // fewer keys than k_rem (cannot happen for finite input)
            Trel |= static_cast<unsigned long long>(r.digit) << shift;
            k_rem -= r.above;
            done = r.count == k_rem;       // whole bucket taken: lower digits stay 0
            shift_prev = shift;
        }
        T = base + Trel;
    }
    if (tid == 0) {
        SelState ns = st;
        ns.T = T;
        ns.k_rem = k_rem;
        ns.done = 1;
        ns.lo = lo;
        ns.span = span;
        state[l] = ns;
        publish_threshold(pred, l, L.large, L.k, T);
    }
}

// ----------------------------------------------------------------- mark --
// OR a 64-bit group of mask bits that starts at bit position pos into a bitmask whose
// words may be shared with other workgroups (rows that are not a multiple of 32 long).
__device__ __forceinline__ void or_bits_shared(uint32_t *__restrict__ mask, size_t pos,
                                               unsigned long long v) {
    if (!v) return;
    const size_t w = pos >> 5;
    const uint32_t b = static_cast<uint32_t>(pos & 31);
    const uint32_t p0 = static_cast<uint32_t>(v << b);
    const uint32_t p1 = static_cast<uint32_t>(b ? (v >> (32 - b)) : (v >> 32));
    const uint32_t p2 = b ? static_cast<uint32_t>(v >> (64 - b)) : 0u;
    if (p0) atomicOr(&mask[w], p0);
    if (p1) atomicOr(&mask[w + 1], p1);
    if (p2) atomicOr(&mask[w + 2], p2);
}
// Full-map layers: workgroups stride over the 16 x 256 tiles (the NSI tiling).  Every centre
// of a tile and of a halo of h rows / columns is compared with the layer's threshold; the
// per-row results become 64-bit ballot words in LDS, the p x p box dilation (Section III-C:
// whole neighbourhoods are kept) is done on those words with shifts and ORs, and the tile's
// mask words are written with plain stores (rows that are a multiple of 32 long) -- no
// global atomics on that path.
// The first n_bucket_wgs workgroups take the layers on the candidate path, one workgroup per
// layer and shard of the layer's threshold-bucket list: the recorded candidates above the bucket
// were marked by the gather pass, those of the bucket that reach the threshold are marked here,
// each ORing the bits of its window into the mask.  (One workgroup per layer doing this at the
// end of k_finish took 20 .. 75 us: the marks of a large layer are too many for one CU.)  The
// next n_list_wgs workgroups stride over the plan's list of tiles of the layers that are
// always ranked on the full map; the others run only when some large layer fell back to it,
// walk all tiles and take those of such layers.
constexpr int kMarkCountSlots = 64;   // chunks a tile counts for in LDS (more only for rows beyond 32 K elements: directly)

struct MarkArgs {
    const LayerDev *layers;
    const SelState *state;
    uint32_t n_bucket_wgs;           // n_layers * kListShards
    const uint32_t *list_cnt;
    const unsigned long long *list_ent;
    const uint32_t *slot_cnt;
    const unsigned long long *slot_ent;
    const DirEntry *dir;             // tiles of all layers in layer order (fallback walk)
    uint32_t n_layers, n_tiles;
    const SampleEntry *map_tiles;
    uint32_t n_map_tiles, n_list_wgs;
    const uint32_t *flags;
    const uint32_t *keys;            // score map
    uint32_t *mask, *cmask;
    uint32_t *chunk_cnt, *group_cnt; // kept elements per chunk / chunk group, counted as the bits are set
};

template <bool COUNT>
__global__ __launch_bounds__(256) void k_mark(const MarkArgs m) {
    constexpr int MAXH = (RSDGC_MAX_P - 1) / 2;
    constexpr int NSEG = kTileCols / 64;       // 64-column segments of a tile row
    static_assert(kTileRows * NSEG == 64, "one lane of wave 0 per row segment");
    __shared__ unsigned long long bits[kTileRows + 2 * MAXH][NSEG + 2];   // [row][left, segments, right]
    __shared__ uint32_t ccnt[kMarkCountSlots];      // bits set by the tile, per chunk from the tile's first one on
    const LayerDev *__restrict__ layers = m.layers;
    const DirEntry *__restrict__ dir = m.dir;
    const SampleEntry *__restrict__ map_tiles = m.map_tiles;
    const SelState *__restrict__ state = m.state;
    const uint32_t *__restrict__ keys = m.keys;
    uint32_t *__restrict__ mask = m.mask;
    uint32_t *__restrict__ cmask = m.cmask;
    const uint32_t n_layers = m.n_layers;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (blockIdx.x < m.n_bucket_wgs) {
        const uint32_t l = blockIdx.x / kListShards, shard = blockIdx.x % kListShards;
        const uint32_t *__restrict__ cnt = m.list_cnt + static_cast<size_t>(l) * kListShards * kListCntStride;
        const uint32_t c = static_cast<uint32_t>(lane) < kListShards ? cnt[lane * kListCntStride] : 0u;
        const SelState st = state[l];
        if (st.mode != kModeCandidates || st.span == 0u) return;      // (no bucket: nothing was ranked)
        const LayerDev Lc = layers[l];
        const unsigned long long Tc = st.T;
        const WindowGeom geom = {static_cast<size_t>(Lc.elem_off), static_cast<int>(Lc.R), static_cast<int>(Lc.C),
                                 (static_cast<int>(Lc.p) - 1) / 2};
        const uint32_t shards = Lc.list_shards, cap = Lc.list_cap / shards;
        if (shard >= shards) return;
        const CountCtx cctx = count_ctx(Lc, m.chunk_cnt, m.group_cnt);
        if (__ballot(c > cap) == 0ull) {       // every shard fits: this workgroup takes its shard
            const uint32_t n = __shfl(c, static_cast<int>(shard), 64);
            const unsigned long long *__restrict__ part = m.list_ent + Lc.list_off + static_cast<size_t>(shard) * cap;
            for (uint32_t i = tid; i < n; i += 256) {
                const unsigned long long K = part[i];
                if (K >= Tc) mark_window<COUNT>(geom, cctx, ~static_cast<uint32_t>(K), mask, cmask);
            }
        } else {                               // the list overflowed: the bucket's keys are still in the tile slots
            const unsigned long long bucket_end = (static_cast<unsigned long long>(st.lo) + (1ull << st.span)) << 32;
            for (uint32_t t = shard; t < Lc.n_tiles; t += shards) {
                const uint32_t n = min(m.slot_cnt[Lc.tile_begin_all + t], Lc.slot_cap);
                const unsigned long long *__restrict__ ent = m.slot_ent + Lc.slot_off + static_cast<size_t>(t) * Lc.slot_cap;
                for (uint32_t i = tid; i < n; i += 256) {
                    const unsigned long long K = ent[i];
                    if (K >= Tc && K < bucket_end) mark_window<COUNT>(geom, cctx, ~static_cast<uint32_t>(K), mask, cmask);
                }
            }
        }
        return;
    }
    const uint32_t bid = blockIdx.x - m.n_bucket_wgs;
    const bool listed = bid < m.n_list_wgs;
    const uint32_t first = listed ? bid : bid - m.n_list_wgs;
    const uint32_t stride = listed ? m.n_list_wgs : gridDim.x - m.n_bucket_wgs - m.n_list_wgs;
    const uint32_t n_items = listed ? m.n_map_tiles : m.n_tiles;
    if (first >= n_items) return;
    if (!listed && m.flags[0] == 0u) return;
    if (COUNT && tid < kMarkCountSlots) ccnt[tid] = 0u;       // (the tile loop's barriers come before the first use)
    uint32_t e = listed ? 0u : dir_lookup(dir, n_layers, first);
    uint32_t cur_l = 0xffffffffu;
    bool active = false;
    unsigned long long T = 0;
    LayerDev L;
    for (uint32_t t = first; t < n_items; t += stride) {
        uint32_t l, local;
        if (listed) {
            const SampleEntry se = map_tiles[t];
            l = se.layer;
            local = se.local_tile;
        } else {
            e = dir_advance(dir, n_layers, e, t);
            l = dir[e].layer;
            local = t - dir[e].begin;
        }
        if (l != cur_l) {
            cur_l = l;
            L = layers[l];
            const SelState st = state[l];
            active = st.mode == kModeFullMap && (listed || L.large != 0u);
            T = st.T;
        }
        if (!active) {
            if (!listed) {
                const uint32_t nb = dir[e + 1].begin;
                t += (nb - t + stride - 1) / stride * stride - stride;
            }
            continue;
        }
        const int h = (static_cast<int>(L.p) - 1) / 2;
        const int rows_ext = kTileRows + 2 * h;
        const int trow = static_cast<int>(local / L.tiles_x);
        const int tcol = static_cast<int>(local - static_cast<uint32_t>(trow) * L.tiles_x);
        const int R = static_cast<int>(L.R), C = static_cast<int>(L.C);
        const int x0 = trow * kTileRows, y0 = tcol * kTileCols;
        const uint32_t *__restrict__ src = keys + L.elem_off;
        const CountCtx cctx = count_ctx(L, m.chunk_cnt, m.group_cnt);
        const uint32_t cl0 = static_cast<uint32_t>((static_cast<size_t>(x0) * C + y0) / kChunk);   // the tile's first chunk

        // wave w takes segment w of every row: all its keys are requested before any is compared
        static_assert(NSEG == 4, "one wave per 64-column segment");
        constexpr int kMaxRowsExt = kTileRows + 2 * MAXH;
        {
            const int y = y0 + 64 * wave + lane;
            uint32_t key[kMaxRowsExt];
#pragma unroll
            for (int rr = 0; rr < kMaxRowsExt; ++rr) {
                const int x = x0 - h + rr;
                key[rr] = 0;
                if (rr < rows_ext && x >= 0 && x < R && y < C)
                    key[rr] = src[static_cast<uint32_t>(x) * L.C + static_cast<uint32_t>(y)];
            }
#pragma unroll
            for (int rr = 0; rr < kMaxRowsExt; ++rr) {
                const int x = x0 - h + rr;
                bool flag = false;
                if (rr < rows_ext && x >= 0 && x < R && y < C) {
                    const uint32_t i = static_cast<uint32_t>(x) * L.C + static_cast<uint32_t>(y);
                    flag = composite_key(key[rr], i) >= T;
                }
                const unsigned long long w = __ballot(flag);
                if (lane == 0 && rr < rows_ext) bits[rr][1 + wave] = w;
            }
        }
        if (wave < 2 && lane < rows_ext) {      // halo columns: lane = row; wave 0 left, wave 1 right
            unsigned long long hw = 0;
            const int x = x0 - h + lane;
            if (x >= 0 && x < R) {
                for (int d = 1; d <= h; ++d) {
                    const int y = wave == 0 ? y0 - d : y0 + kTileCols + (d - 1);
                    if (y >= 0 && y < C) {
                        const uint32_t i = static_cast<uint32_t>(x) * L.C + static_cast<uint32_t>(y);
                        if (composite_key(src[i], i) >= T)
                            hw |= wave == 0 ? (1ull << (64 - d)) : (1ull << (d - 1));
                    }
                }
            }
            bits[lane][wave == 0 ? 0 : NSEG + 1] = hw;
        }
        __syncthreads();

        const int r = lane / NSEG, seg = lane % NSEG;    // wave 0: rows x segments = 64 items
        const int x = x0 + r, yb = y0 + 64 * seg;
        if (wave == 0 && x < R && yb < C) {
            unsigned long long acc = 0;
            for (int rr = r; rr <= r + 2 * h; ++rr) {
                const unsigned long long W = bits[rr][1 + seg], Lw = bits[rr][seg], Rw = bits[rr][2 + seg];
                unsigned long long hd = W;
                for (int d = 1; d <= h; ++d)
                    hd |= (W << d) | (Lw >> (64 - d)) | (W >> d) | (Rw << (64 - d));
                acc |= hd;
            }
            const int ncols = min(64, C - yb);
            const unsigned long long valid = ncols >= 64 ? ~0ull : ((1ull << ncols) - 1ull);
            acc &= valid;
            const unsigned long long own = bits[r + h][1 + seg];
            const size_t pos = static_cast<size_t>(L.elem_off) + static_cast<size_t>(x) * C + yb;
            if ((C & 31) == 0) {                     // the tile owns its mask words
                const size_t w = pos >> 5;
                mask[w] = static_cast<uint32_t>(acc);
                if (ncols > 32) mask[w + 1] = static_cast<uint32_t>(acc >> 32);
                if (cmask) {
                    cmask[w] = static_cast<uint32_t>(own);
                    if (ncols > 32) cmask[w + 1] = static_cast<uint32_t>(own >> 32);
                }
                // its bits, per chunk (the two words may lie in different chunks)
#pragma unroll
                for (int part = 0; part < 2; ++part) {
                    const uint32_t n = COUNT ? __popc(static_cast<uint32_t>(acc >> (32 * part))) : 0u;
                    if (n) {
                        const uint32_t slot = static_cast<uint32_t>((w + part - cctx.word0) >> 8) - cl0;
                        if (slot < static_cast<uint32_t>(kMarkCountSlots)) atomicAdd(&ccnt[slot], n);
                        else count_add_chunk(cctx, cl0 + slot, n);
                    }
                }
            } else if (!COUNT) {
                or_bits_shared(mask, pos, acc);
                if (cmask) or_bits_shared(cmask, pos, own);
            } else {                                 // shared words: an OR tells which bits were new
                const size_t w = pos >> 5;
                const uint32_t b = static_cast<uint32_t>(pos & 31);
                const uint32_t part[3] = {static_cast<uint32_t>(acc << b),
                                          static_cast<uint32_t>(b ? (acc >> (32 - b)) : (acc >> 32)),
                                          b ? static_cast<uint32_t>(acc >> (64 - b)) : 0u};
#pragma unroll
                for (int j = 0; j < 3; ++j) {
                    if (part[j] == 0u) continue;
                    const uint32_t n = __popc(part[j] & ~atomicOr(&mask[w + j], part[j]));
                    if (n) {
                        const uint32_t slot = static_cast<uint32_t>((w + j - cctx.word0) >> 8) - cl0;
                        if (slot < static_cast<uint32_t>(kMarkCountSlots)) atomicAdd(&ccnt[slot], n);
                        else count_add_chunk(cctx, cl0 + slot, n);
                    }
                }
                if (cmask) or_bits_shared(cmask, pos, own);
            }
        }
        __syncthreads();                        // the ballot words are reused by the next tile
        static_assert(kMarkCountSlots == 64, "one lane of the first wave per counted chunk");
        if (COUNT && tid < 64) {
            count_flush_wave0(cctx, cl0, ccnt[tid]);
            ccnt[tid] = 0u;
        }
    }
}

// ---------------------------------------------------------------- count --
// Kept elements (and selected centres) per chunk and per group of kChunkGroup chunks, from the
// finished masks -- for plans of many chunks; a small plan's kept elements are counted where their
// bits are set (CountCtx) and `mask` is null here.  One workgroup per kCountChunks = 16 chunks; 16 adjacent threads read the 256 mask words of one
// chunk (16 consecutive words each, as independent 8-byte loads) and add their popcounts with
// four shuffles.  A workgroup adds its total to its chunk group's with one atomic -- four per
// group (one atomic per chunk put 17 k of them on 9 cache lines and cost 18 us).
constexpr int kCountThreads = 16 * kCountChunks;

__global__ __launch_bounds__(kCountThreads) void k_count(const CountGroup *__restrict__ groups,
                                                         const uint32_t *__restrict__ mask,
                                                         const uint32_t *__restrict__ cmask,
                                                         uint32_t *__restrict__ chunk_cnt,
                                                         uint32_t *__restrict__ chunk_ccnt,
                                                         uint32_t *__restrict__ group_cnt,
                                                         uint32_t *__restrict__ group_ccnt, uint32_t gstride) {
    constexpr int kPerThread = kChunk / 32 / 16;    // 16 words
    static_assert(kCountChunks <= 64, "one lane of the first wave per chunk");
    __shared__ uint32_t lcnt[2][kCountChunks];
    const int tid = threadIdx.x;
    const CountGroup gr = groups[blockIdx.x];
    const uint32_t i0 = static_cast<uint32_t>(tid) * kPerThread;
    // (a layer starts at a multiple of 64 elements, so word0 and i0 are even: 8-byte loads)
    uint2 wa[kPerThread / 2], wb[kPerThread / 2];
#pragma unroll
    for (int j = 0; j < kPerThread / 2; ++j) {
        const uint32_t i = i0 + 2 * j;
        wa[j] = make_uint2(0u, 0u);
        wb[j] = make_uint2(0u, 0u);
        if (i + 1 < gr.n_words) {
            if (mask) wa[j] = *reinterpret_cast<const uint2 *>(mask + gr.word0 + i);
            if (cmask) wb[j] = *reinterpret_cast<const uint2 *>(cmask + gr.word0 + i);
        } else if (i < gr.n_words) {
            if (mask) wa[j].x = mask[gr.word0 + i];
            if (cmask) wb[j].x = cmask[gr.word0 + i];
        }
    }
    uint32_t a = 0, b = 0;
#pragma unroll
    for (int j = 0; j < kPerThread / 2; ++j) {
        a += __popc(wa[j].x) + __popc(wa[j].y);
        b += __popc(wb[j].x) + __popc(wb[j].y);
    }
#pragma unroll
    for (int d = 8; d >= 1; d >>= 1) {
        a += __shfl_xor(a, d, 64);
        b += __shfl_xor(b, d, 64);
    }
    if ((tid & 15) == 0) {
        lcnt[0][tid >> 4] = a;
        lcnt[1][tid >> 4] = b;
    }
    __syncthreads();
    if (tid < 64) {                        // the first wave: one lane per chunk
        a = tid < kCountChunks ? lcnt[0][tid] : 0u;
        b = tid < kCountChunks ? lcnt[1][tid] : 0u;
        if (static_cast<uint32_t>(tid) < gr.n_chunks) {
            if (mask) chunk_cnt[gr.first_chunk + tid] = a;
            if (cmask) chunk_ccnt[gr.first_chunk + tid] = b;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            a += __shfl_xor(a, d, 64);
            b += __shfl_xor(b, d, 64);
        }
        if (tid == 0) {                    // (the group totals are cleared at the start of the call)
            if (mask && a) atomicAdd(&group_cnt[static_cast<size_t>(gr.group) * gstride], a);
            if (cmask && b) atomicAdd(&group_ccnt[static_cast<size_t>(gr.group) * gstride], b);
        }
    }
}

// The chunk's prefix -- kept elements of its layer before it -- is the sum of the totals of
// the layer's earlier chunk groups and of the earlier chunks of its own group: at most a few
// hundred values, so every consumer adds them up itself instead of waiting for a scan
// kernel.  The first wave does it (independent loads issued with the workgroup's other loads,
// one wave reduction) and leaves the sum in *s_prefix; the caller reads it after its next
// barrier.
__device__ __forceinline__ uint32_t chunk_prefix_by_wave(const ChunkInfo &ci, uint32_t c,
                                                         const uint32_t *__restrict__ chunk_cnt,
                                                         const uint32_t *__restrict__ group_cnt) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t g0 = ci.layer_first_group + lane, g1 = ci.group;
    const uint32_t cc = ci.group_first_chunk + lane;     // at most kChunkGroup - 1 = 63 of them
    uint32_t v[5];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = g0 + 64 * j < g1 ? group_cnt[static_cast<size_t>(g0 + 64 * j) * ci.gstride] : 0u;
    v[4] = cc < c ? chunk_cnt[cc] : 0u;
    uint32_t own = v[0] + v[1] + v[2] + v[3] + v[4];
    for (uint32_t g = g0 + 256; g < g1; g += 64) own += group_cnt[static_cast<size_t>(g) * ci.gstride];     // layers beyond 2^27 elements
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) own += __shfl_xor(own, d, 64);
    return own;                    // the same in every lane of the wave
}

__device__ __forceinline__ void chunk_prefix_wave0(const ChunkInfo &ci, uint32_t c,
                                                   const uint32_t *__restrict__ chunk_cnt,
                                                   const uint32_t *__restrict__ group_cnt,
                                                   uint32_t *s_prefix) {
    if (threadIdx.x >= 64) return;
    const uint32_t own = chunk_prefix_by_wave(ci, c, chunk_cnt, group_cnt);
    if (threadIdx.x == 0) *s_prefix = own;
}

// ----------------------------------------------------------------- emit --
// Streams g and r once more: v = r + g; kept elements go out in ascending index order at
// the position given by the chunk prefix plus the popcount of the mask bits before them;
// the residual becomes +0 where kept and v elsewhere.
__global__ __launch_bounds__(256) void k_emit(const LayerDev *__restrict__ layers,
                                              const ChunkInfo *__restrict__ chunk_info, const float *__restrict__ grad,
                                              float *__restrict__ resid,
                                              const uint32_t *__restrict__ mask,
                                              const uint32_t *__restrict__ chunk_cnt,
                                              const uint32_t *__restrict__ group_cnt,
                                              uint32_t *__restrict__ out_idx,
                                              float *__restrict__ out_val,
                                              int32_t *__restrict__ out_counts) {
    __shared__ uint32_t wave_tot[4];
    __shared__ uint32_t s_word[256];
    __shared__ uint32_t s_pref[256];
    __shared__ uint32_t s_cbase;
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const ChunkInfo ci = chunk_info[c];
    const LayerDev L = layers[ci.layer];
    const uint32_t start = ci.start, len = ci.len;
    const size_t base = ci.arena_off;
    const uint32_t nwords = (len + 31) >> 5;
    const uint32_t word = static_cast<uint32_t>(tid) < nwords ? mask[(base >> 5) + tid] : 0;
    const float *__restrict__ g = grad + base;
    float *__restrict__ r = resid + base;
    const bool whole = len == static_cast<uint32_t>(kChunk);
    // A whole chunk: every load is issued before the mask scan, so the scan's latency and the
    // loads overlap and each thread keeps 16 wide loads in flight.
    float4 gq[kChunk / 1024], rq[kChunk / 1024];
    if (whole) {
#pragma unroll
        for (int j = 0; j < kChunk / 1024; ++j) {
            gq[j] = load_streaming(g + j * 1024 + 4 * tid);
            rq[j] = load_streaming(r + j * 1024 + 4 * tid);
        }
    }
    chunk_prefix_wave0(ci, c, chunk_cnt, group_cnt, &s_cbase);
    const uint32_t cnt = __popc(word);
    s_word[tid] = word;
    const uint32_t incl = block_scan_incl(cnt, wave_tot);
    const uint32_t cbase = s_cbase;
    const size_t obase = static_cast<size_t>(L.out_off) + cbase;
    const uint32_t room = L.cap > cbase ? L.cap - cbase : 0u;   // never write past the segment
    s_pref[tid] = incl - cnt;
    if (ci.last && tid == 255) out_counts[ci.layer] = static_cast<int32_t>(cbase + incl);
    __syncthreads();
    if (whole) {
#pragma unroll
        for (int j = 0; j < kChunk / 1024; ++j) {
            const uint32_t e = j * 1024 + 4 * tid;
            const uint32_t w = s_word[e >> 5];
            const uint32_t sh = e & 31;
            const uint32_t bits = (w >> sh) & 0xfu;
            float v[4] = {rq[j].x + gq[j].x, rq[j].y + gq[j].y, rq[j].z + gq[j].z, rq[j].w + gq[j].w};
            if (bits) {
                uint32_t pos = s_pref[e >> 5] + __popc(w & ((1u << sh) - 1u));
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (bits & (1u << q)) {
                        if (pos < room) {
                            out_idx[obase + pos] = start + e + q;
                            out_val[obase + pos] = v[q];
                        }
                        ++pos;
                        v[q] = 0.f;
                    }
            }
            store_streaming(r + e, make_float4(v[0], v[1], v[2], v[3]));
        }
        return;
    }
#pragma unroll 2
    for (int j = 0; j < kChunk / 1024; ++j) {
        const uint32_t e = j * 1024 + 4 * tid;
        if (e >= len) break;
        const uint32_t w = s_word[e >> 5];
        const uint32_t sh = e & 31;
        const uint32_t bits = (w >> sh) & 0xfu;
        if (e + 3 < len) {
            const float4 gv = *reinterpret_cast<const float4 *>(g + e);
            const float4 rv = *reinterpret_cast<const float4 *>(r + e);
            float v[4] = {rv.x + gv.x, rv.y + gv.y, rv.z + gv.z, rv.w + gv.w};
            if (bits) {
                uint32_t pos = s_pref[e >> 5] + __popc(w & ((1u << sh) - 1u));
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (bits & (1u << q)) {
                        if (pos < room) {
                            out_idx[obase + pos] = start + e + q;
                            out_val[obase + pos] = v[q];
                        }
                        ++pos;
                        v[q] = 0.f;
                    }
            }
            *reinterpret_cast<float4 *>(r + e) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
            uint32_t pos = s_pref[e >> 5] + __popc(w & ((1u << sh) - 1u));
            for (uint32_t q = 0; q < 4 && e + q < len; ++q) {
                float v = r[e + q] + g[e + q];
                if (bits & (1u << q)) {
                    if (pos < room) {
                        out_idx[obase + pos] = start + e + q;
                        out_val[obase + pos] = v;
                    }
                    ++pos;
                    v = 0.f;
                }
                r[e + q] = v;
            }
        }
    }
}

// Two-buffer form of the emit: the NSI passes have already stored v = r + g in the second
// residual arena, so only the kept elements are touched -- their value goes out and the
// arena gets +0 there.  A chunk without kept elements costs one read of its mask words.  A
// layer with k_l = 0 went through no NSI pass; its v is formed here.
// (Four chunks per workgroup -- a quarter of the dependent chains of mask word, prefix and kept
// values, four value requests per thread in flight -- was built and measured: no faster.  The
// kernel is bound by the rate of its scattered 4-byte reads and writes, not by their latency.)
__global__ __launch_bounds__(256) void k_emit_sparse(const ChunkInfo *__restrict__ chunk_info,
                                                     const SelState *__restrict__ state,
                                                     const float *__restrict__ grad,
                                                     const float *__restrict__ resid_in,
                                                     float *__restrict__ v_arena,
                                                     const float *__restrict__ mom_in,
                                                     float *__restrict__ mom_arena, float m,
                                                     const uint32_t *__restrict__ mask,
                                                     const uint32_t *__restrict__ chunk_cnt,
                                                     const uint32_t *__restrict__ group_cnt,
                                                     uint32_t *__restrict__ out_idx,
                                                     float *__restrict__ out_val,
                                                     int32_t *__restrict__ out_counts) {
    __shared__ uint32_t wave_tot[4];
    __shared__ uint16_t s_list[kChunk];
    __shared__ uint32_t s_total, s_cbase;
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const ChunkInfo ci = chunk_info[c];
    const uint32_t start = ci.start, len = ci.len;
    const size_t base = ci.arena_off;
    float *__restrict__ v = v_arena + base;
    // the three loads that depend only on the chunk's entry go out together
    const uint32_t nwords = (len + 31) >> 5;
    uint32_t word = static_cast<uint32_t>(tid) < nwords ? mask[(base >> 5) + tid] : 0;
    const uint32_t mode = state[ci.layer].mode;
    chunk_prefix_wave0(ci, c, chunk_cnt, group_cnt, &s_cbase);
    if (mode == kModeSkip) {
        if (ci.last && tid == 0) out_counts[ci.layer] = 0;
        const float *__restrict__ g = grad + base;
        const float *__restrict__ r = resid_in + base;
        for (uint32_t e = 4 * tid; e < len; e += 1024) {
            for (uint32_t q = 0; q < 4 && e + q < len; ++q) {
                float gu = g[e + q];
                if (mom_in) {
                    gu = __fmul_rn(m, mom_in[base + e + q]) + gu;
                    mom_arena[base + e + q] = gu;
                }
                v[e + q] = r[e + q] + gu;
            }
        }
        return;
    }
    if (!__syncthreads_or(word != 0u) && !ci.last) return;      // uniform
    const uint32_t cbase = s_cbase;
    const uint32_t cnt = __popc(word);
    const uint32_t incl = block_scan_incl(cnt, wave_tot);
    // the chunk's kept elements, in ascending order, as offsets inside the chunk
    uint32_t pos = incl - cnt;
    while (word) {
        const uint32_t b = static_cast<uint32_t>(__ffs(word)) - 1u;
        word &= word - 1u;
        s_list[pos++] = static_cast<uint16_t>(32u * static_cast<uint32_t>(tid) + b);
    }
    if (tid == 255) {
        s_total = incl;
        if (ci.last) out_counts[ci.layer] = static_cast<int32_t>(cbase + incl);
    }
    __syncthreads();
    const uint32_t total = s_total;
    const size_t obase = static_cast<size_t>(ci.out_off) + cbase;
    const uint32_t room = ci.cap > cbase ? ci.cap - cbase : 0u;   // never write past the segment
    // one kept element per thread: independent loads, coalesced pair stores
    for (uint32_t i = tid; i < total; i += 256) {
        const uint32_t e = s_list[i];
        if (e >= len) break;                // (mask bits exist only for elements of the layer)
        const float val = v[e];
        if (i < room) {
            out_idx[obase + i] = start + e;
            out_val[obase + i] = val;
        }
        v[e] = 0.f;
        if (mom_arena) mom_arena[base + e] = 0.f;     // the momentum restarts where v was sent
    }
}

// Ascending list of the selected centres of every layer.
__global__ __launch_bounds__(256) void k_emit_centres(const LayerDev *__restrict__ layers,
                                                      const ChunkInfo *__restrict__ chunk_info,
                                                      const uint32_t *__restrict__ cmask,
                                                      const uint32_t *__restrict__ chunk_ccnt,
                                                      const uint32_t *__restrict__ group_ccnt,
                                                      uint32_t *__restrict__ out_centre_idx,
                                                      int32_t *__restrict__ out_centre_counts) {
    __shared__ uint32_t wave_tot[4];
    __shared__ uint32_t s_cbase;
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const ChunkInfo ci = chunk_info[c];
    const LayerDev L = layers[ci.layer];
    const uint32_t start = ci.start;
    const size_t base = ci.arena_off;
    const uint32_t nwords = (ci.len + 31) >> 5;
    uint32_t word = static_cast<uint32_t>(tid) < nwords ? cmask[(base >> 5) + tid] : 0;
    chunk_prefix_wave0(ci, c, chunk_ccnt, group_ccnt, &s_cbase);
    const uint32_t cnt = __popc(word);
    const uint32_t incl = block_scan_incl(cnt, wave_tot);
    const uint32_t cbase = s_cbase;
    if (ci.last && tid == 255 && out_centre_counts) out_centre_counts[ci.layer] = static_cast<int32_t>(cbase + incl);
    uint32_t rank = cbase + (incl - cnt);
    while (word) {
        const int b = __ffs(word) - 1;
        word &= word - 1;
        if (out_centre_idx && rank < L.k) out_centre_idx[static_cast<size_t>(L.centre_off) + rank] = start + 32u * tid + b;
        ++rank;
    }
}

// ----------------------------------------------------------- decompress --
// +0 into every element of every layer (the padding between layers is left alone): one chunk
// per workgroup, streaming 16-byte stores.
__global__ __launch_bounds__(256) void k_zero_layers(const ChunkInfo *__restrict__ chunk_info, float *__restrict__ dense) {
    const int tid = threadIdx.x;
    const ChunkInfo ci = chunk_info[blockIdx.x];
    const uint32_t len = ci.len;
    float *__restrict__ d = dense + ci.arena_off;
#pragma unroll
    for (int j = 0; j < kChunk / 1024; ++j) {
        const uint32_t e = j * 1024 + 4 * tid;
        if (e >= len) break;
        if (e + 3 < len) {
            store_streaming(d + e, make_float4(0.f, 0.f, 0.f, 0.f));
        } else {
            for (uint32_t q = 0; q < 4 && e + q < len; ++q) d[e + q] = 0.f;
        }
    }
}

__global__ __launch_bounds__(256) void k_scatter(const LayerDev *__restrict__ layers, int n_layers,
                                                 long long capacity,
                                                 const uint32_t *__restrict__ idx,
                                                 const float *__restrict__ val,
                                                 const int32_t *__restrict__ counts,
                                                 float *__restrict__ dense, int accumulate) {
    const long long j = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
    if (j >= capacity) return;
    int lo = 0, hi = n_layers;            // last layer whose segment starts at or before j
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (layers[mid].out_off <= j) lo = mid; else hi = mid;
    }
    const LayerDev L = layers[lo];
    const long long q = j - L.out_off;
    if (q >= counts[lo] || q >= static_cast<long long>(L.cap)) return;
    const uint32_t i = idx[j];
    if (i >= L.G) return;                 // malformed message: ignore the pair
    float *d = dense + L.elem_off + i;
    if (accumulate) *d = *d + val[j]; else *d = val[j];
}

// --------------------------------------------------------- block reading --
// Non-overlapping p x p neighbourhoods (the other reading of Section III-C): one score per
// block.  `outer` are the element matrices, `inner` the block grids (one "element" per block).
// Work unit: a tile of 8 block rows by block_tile_cols(P) block columns of one layer.  Its
// elements are loaded with 16-byte loads (rows that are a multiple of 4 floats long), v = r + g
// goes to LDS and to the new residual arena (which may be r's own: no element is read by two
// tiles), then every thread takes blocks of the tile: Eqs. 8-10 in double over the p*p slots
// (zero outside the matrix, divisor p*p), score to the inner score map, 12-bit histogram.
// Persistent workgroups stride over the tiles; the histogram is flushed on layer change.
// FEED: tiles come from the launch's work feed (many tiles per workgroup) instead of a
// fixed strided share.  MOM: Eq. 12's first line on the way in -- u_new = m*u + g (one rounded
// multiply, one rounded add) takes g's place and goes to the new momentum arena (which, like
// the residual's, may be the old one).
template <int P, bool FEED, bool MOM>
__global__ __launch_bounds__(256) void k_block_nsi(const LayerDev *__restrict__ outer,
                                                   const DirEntry *__restrict__ tile_dir,
                                                   uint32_t n_layers, uint32_t n_tiles,
                                                   const LayerDev *__restrict__ inner,
                                                   const float *__restrict__ grad,
                                                   const float *resid, float *v_out,
                                                   float *__restrict__ score_map,
                                                   uint32_t *__restrict__ hist, double alpha,
                                                   uint32_t *__restrict__ feed_ctr, uint32_t feed_shift,
                                                   const float *mom_in, float *mom_out, float m) {
    constexpr int BCT = block_tile_cols(P);
    constexpr int TR = kBlockTileRows * P, TC = BCT * P;      // tile in elements; TC is a multiple of 4
    constexpr int VEC_PER_ROW = TC / 4;
    constexpr int NVEC = TR * VEC_PER_ROW;
    constexpr int ITER = (NVEC + 255) / 256;
    constexpr int NBLK = kBlockTileRows * BCT;
    static_assert(TC % 4 == 0, "tile rows are whole 16-byte groups");
    __shared__ __attribute__((aligned(16))) float tile[TR * TC];
    __shared__ uint32_t lhist[kHistBins];
    __shared__ uint32_t feed_slot[2];
    const int tid = threadIdx.x;
    const uint32_t stride = gridDim.x;
    WorkFeed feed;
    uint32_t first;
    if (FEED) {
        first = feed.first(feed_ctr, n_tiles, feed_shift, feed_slot);
        if (first == kNoItem) return;      // uniform
    } else {
        first = blockIdx.x;
        if (first >= n_tiles) return;
    }
    for (int b = tid; b < kHistBins; b += 256) lhist[b] = 0;
    __syncthreads();
    const double n = static_cast<double>(P * P);
    const double ca = alpha / n, cb = (1.0 - alpha) / n;
    uint32_t e = dir_lookup(tile_dir, n_layers, first);
    uint32_t cur_l = 0xffffffffu;
    bool active = false;
    LayerDev O, I;
    for (uint32_t t = first; FEED ? t != kNoItem : t < n_tiles;
         t = FEED ? feed.next(feed_slot) : t + stride) {
        e = dir_advance(tile_dir, n_layers, e, t);
        const uint32_t l = tile_dir[e].layer;
        if (l != cur_l) {
            if (active) {                              // flush the finished layer's counts
                uint32_t *__restrict__ gh = hist + static_cast<size_t>(cur_l) * kHistBins;
                for (int b = tid; b < kHistBins; b += 256) {
                    const uint32_t c = lhist[b];
                    if (c) { atomicAdd(&gh[b], c); lhist[b] = 0; }
                }
                __syncthreads();
            }
            cur_l = l;
            O = outer[l];
            I = inner[l];
            active = static_cast<int>(O.p) == P;       // another launch takes the other neighbourhood sides
        }
        if (!active) {
            if (!FEED) {
                const uint32_t nb = tile_dir[e + 1].begin;
                t += (nb - t + stride - 1) / stride * stride - stride;
            }
            continue;
        }
        const uint32_t local = t - tile_dir[e].begin;
        const int trow = static_cast<int>(local / O.tiles_x);
        const int tcol = static_cast<int>(local - static_cast<uint32_t>(trow) * O.tiles_x);
        const int R = static_cast<int>(O.R), C = static_cast<int>(O.C);
        const int x0 = trow * TR, y0 = tcol * TC;
        const float *__restrict__ g = grad + O.elem_off;
        const float *r = resid + O.elem_off;           // may be the same arena as vo
        float *vo = v_out + O.elem_off;
        const float *ui = MOM ? mom_in + O.elem_off : nullptr;     // may be the same arena as uo
        float *uo = MOM ? mom_out + O.elem_off : nullptr;
        if ((C & 3) == 0) {
            float4 gv[ITER], rv[ITER], uv[MOM ? ITER : 1];
#pragma unroll
            for (int it = 0; it < ITER; ++it) {
                const int s = tid + it * 256;
                const int rr = s / VEC_PER_ROW, j4 = s - rr * VEC_PER_ROW;
                const int x = x0 + rr, y = y0 + 4 * j4;
                gv[it] = make_float4(0.f, 0.f, 0.f, 0.f);
                rv[it] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (MOM) uv[it] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (s < NVEC && x < R && y < C) {
                    const size_t off = static_cast<size_t>(x) * C + y;
                    gv[it] = load_streaming(g + off);       // blocks share no element
                    rv[it] = load_streaming(r + off);
                    if (MOM) uv[it] = load_streaming(ui + off);
                }
            }
            if (FEED) feed.stash(feed_slot);      // the loads are out, no store of this tile yet
#pragma unroll
            for (int it = 0; it < ITER; ++it) {
                const int s = tid + it * 256;
                if (s < NVEC) {
                    const int rr = s / VEC_PER_ROW, j4 = s - rr * VEC_PER_ROW;
                    const int x = x0 + rr, y = y0 + 4 * j4;
                    const bool inside = x < R && y < C;
                    if (MOM) {
                        gv[it].x = __fmul_rn(m, uv[it].x) + gv[it].x;
                        gv[it].y = __fmul_rn(m, uv[it].y) + gv[it].y;
                        gv[it].z = __fmul_rn(m, uv[it].z) + gv[it].z;
                        gv[it].w = __fmul_rn(m, uv[it].w) + gv[it].w;
                        if (inside) store_streaming(uo + static_cast<size_t>(x) * C + y, gv[it]);
                    }
                    const float4 v = make_float4(rv[it].x + gv[it].x, rv[it].y + gv[it].y,
                                                 rv[it].z + gv[it].z, rv[it].w + gv[it].w);
                    *reinterpret_cast<float4 *>(&tile[s * 4]) = v;          // s*4 == rr*TC + 4*j4
                    if (inside) store_streaming(vo + static_cast<size_t>(x) * C + y, v);
                }
            }
        } else {
            for (int s = tid; s < TR * TC; s += 256) {
                const int rr = s / TC, j = s - rr * TC;
                const int x = x0 + rr, y = y0 + j;
                float v = 0.f;
                if (x < R && y < C) {
                    const size_t off = static_cast<size_t>(x) * C + y;
                    float gu = g[off];
                    if (MOM) {
                        gu = __fmul_rn(m, ui[off]) + gu;
                        uo[off] = gu;
                    }
                    v = r[off] + gu;
                    vo[off] = v;
                }
                tile[s] = v;
            }
        }
        __syncthreads();
        const uint32_t BR = I.R, BC = I.C;
#pragma unroll
        for (int q = tid; q < NBLK; q += 256) {
            const int br = q / BCT, bc = q - br * BCT;
            const uint32_t bx = static_cast<uint32_t>(trow * kBlockTileRows + br);
            const uint32_t by = static_cast<uint32_t>(tcol * BCT + bc);
            if (bx < BR && by < BC) {
                double sa = 0.0, ss = 0.0, sq = 0.0;
#pragma unroll
                for (int dx = 0; dx < P; ++dx)
#pragma unroll
                    for (int dy = 0; dy < P; ++dy) {
                        const double w = static_cast<double>(tile[(br * P + dx) * TC + bc * P + dy]);
                        sa += fabs(w);
                        ss += w;
                        sq = fma(w, w, sq);
                    }
                const double nsq = __dmul_rn(n, sq);
                double d = var_n2_one_pass(ss, nsq);
                if (P > 1 && d < kCancelFrac * nsq)          // the one-pass variance cancelled (rare)
                    d = __dmul_rn(n, window_ssd<P>(&tile[(br * P) * TC + bc * P], TC, ss / n));
                const float score = static_cast<float>(nsi_from_var(sa, d, ca, cb));
                score_map[I.elem_off + static_cast<size_t>(bx) * BC + by] = score;
                atomicAdd(&lhist[(__float_as_uint(score) & 0x7fffffffu) >> 19], 1u);
            }
        }
        __syncthreads();                               // the tile is reused by the next item
    }
    if (active) {
        uint32_t *__restrict__ gh = hist + static_cast<size_t>(cur_l) * kHistBins;
        for (int b = tid; b < kHistBins; b += 256) {
            const uint32_t c = lhist[b];
            if (c) atomicAdd(&gh[b], c);
        }
    }
}

// Kept blocks of one chunk of a layer's grid, in ascending order: block index to the index
// list, the block's p*p values (row-major, +0 for slots outside the matrix) to the value
// list, +0 into the new residual (and into the new momentum, when the call carries one).
__global__ __launch_bounds__(256) void k_emit_blocks(const LayerDev *__restrict__ outer,
                                                     const ChunkInfo *__restrict__ inner_chunks,
                                                     const uint32_t *__restrict__ mask,
                                                     const uint32_t *__restrict__ chunk_cnt,
                                                     const uint32_t *__restrict__ group_cnt,
                                                     const LayerDev *__restrict__ inner,
                                                     float *__restrict__ v_arena,
                                                     float *__restrict__ u_arena /* nullable */,
                                                     uint32_t *__restrict__ out_blocks,
                                                     float *__restrict__ out_val,
                                                     int32_t *__restrict__ out_counts) {
    __shared__ uint32_t wave_tot[4];
    __shared__ uint16_t s_list[kChunk];
    __shared__ uint32_t s_total, s_cbase;
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const ChunkInfo ci = inner_chunks[c];
    const uint32_t nwords = (ci.len + 31) >> 5;
    uint32_t word = static_cast<uint32_t>(tid) < nwords ? mask[(ci.arena_off >> 5) + tid] : 0;
    chunk_prefix_wave0(ci, c, chunk_cnt, group_cnt, &s_cbase);
    if (!__syncthreads_or(word != 0u) && !ci.last) return;      // uniform
    const uint32_t cbase = s_cbase;
    const uint32_t cnt = __popc(word);
    const uint32_t incl = block_scan_incl(cnt, wave_tot);
    uint32_t pos = incl - cnt;
    while (word) {
        const uint32_t b = static_cast<uint32_t>(__ffs(word)) - 1u;
        word &= word - 1u;
        s_list[pos++] = static_cast<uint16_t>(32u * static_cast<uint32_t>(tid) + b);
    }
    if (tid == 255) {
        s_total = incl;
        if (ci.last) out_counts[ci.layer] = static_cast<int32_t>(cbase + incl);
    }
    __syncthreads();
    const uint32_t total = s_total;
    const LayerDev O = outer[ci.layer];
    const int P = static_cast<int>(O.p), R = static_cast<int>(O.R), C = static_cast<int>(O.C);
    const uint32_t BC = inner[ci.layer].C;
    float *__restrict__ v = v_arena + O.elem_off;
    // one thread per (kept block, slot): independent loads, contiguous value stores
    const uint32_t PP = static_cast<uint32_t>(P * P);
    for (uint32_t i = tid; i < total * PP; i += 256) {
        const uint32_t kb = i / PP, sl = i - kb * PP;
        const uint32_t q = s_list[kb];
        if (q >= ci.len) continue;          // (mask bits exist only for blocks of the grid)
        const uint32_t rank = cbase + kb;   // position among the layer's kept blocks
        if (rank >= O.k) continue;          // never write past the layer's segment
        const uint32_t b = ci.start + q;
        const int bx = static_cast<int>(b / BC), by = static_cast<int>(b - static_cast<uint32_t>(bx) * BC);
        if (sl == 0) out_blocks[static_cast<size_t>(O.centre_off) + rank] = b;
        const int dx = static_cast<int>(sl) / P, dy = static_cast<int>(sl) - dx * P;
        const int x = bx * P + dx, y = by * P + dy;
        float val = 0.f;
        if (x < R && y < C) {
            const size_t off = static_cast<size_t>(x) * C + y;
            val = v[off];
            v[off] = 0.f;
            if (u_arena) u_arena[O.elem_off + off] = 0.f;
        }
        out_val[static_cast<size_t>(O.out_off) + static_cast<size_t>(rank) * PP + sl] = val;
    }
}

// Inverse: one thread per kept block of a message.
__global__ __launch_bounds__(256) void k_scatter_blocks(const LayerDev *__restrict__ outer, int n_layers,
                                                        long long capacity,
                                                        const uint32_t *__restrict__ blocks,
                                                        const float *__restrict__ val,
                                                        const int32_t *__restrict__ counts,
                                                        float *__restrict__ dense, int accumulate) {
    const long long j = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
    if (j >= capacity) return;
    int lo = 0, hi = n_layers;            // last layer whose block segment starts at or before j
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (outer[mid].centre_off <= j) lo = mid; else hi = mid;
    }
    const LayerDev O = outer[lo];
    const long long q = j - O.centre_off;
    if (q >= counts[lo] || q >= static_cast<long long>(O.k)) return;
    const int P = static_cast<int>(O.p), R = static_cast<int>(O.R), C = static_cast<int>(O.C);
    const uint32_t BC = (O.C + O.p - 1) / O.p, BR = (O.R + O.p - 1) / O.p;
    const uint32_t b = blocks[j];
    if (b >= BR * BC) return;             // malformed message: ignore the block
    const int bx = static_cast<int>(b / BC), by = static_cast<int>(b - static_cast<uint32_t>(bx) * BC);
    const float *__restrict__ src = val + static_cast<size_t>(O.out_off) + static_cast<size_t>(q) * (P * P);
    float *__restrict__ d = dense + O.elem_off;
    for (int dx = 0; dx < P; ++dx)
        for (int dy = 0; dy < P; ++dy) {
            const int x = bx * P + dx, y = by * P + dy;
            if (x < R && y < C) {
                const size_t off = static_cast<size_t>(x) * C + y;
                if (accumulate) d[off] = d[off] + src[dx * P + dy]; else d[off] = src[dx * P + dy];
            }
        }
}

// ---------------------------------------------------------------- apply --
// Eq. 12, third line: w <- w - eta * (sum over the nodes' messages).  No dense accumulator: the
// messages are index-sorted per layer (rsdgc_compress writes them so), so the pairs that fall into
// one 8192-element chunk of a layer are one contiguous stretch of every message.  A first
// kernel finds those stretches (two binary searches per message and chunk, all in parallel); the
// second takes one chunk per workgroup, sums the messages' values in an LDS array in the order
// given -- message after message, a barrier between them, plain float32 adds starting from +0 --
// and updates the weights at the positions that were named.  One message needs none of this:
// every pair is applied on its own.
struct ApplyMsgs {
    const uint32_t *idx[RSDGC_MAX_MSGS];
    const float *val[RSDGC_MAX_MSGS];
    const int32_t *counts[RSDGC_MAX_MSGS];
};

// First position in a[0, n) whose value is not below x (a ascending).
__device__ __forceinline__ uint32_t lower_bound_u32(const uint32_t *__restrict__ a, uint32_t n, uint32_t x) {
    uint32_t lo = 0, hi = n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ranges[(k * n_chunks + c) * 2 + {0, 1}]: first and one-past-last pair of message k (positions
// in the message's arrays) that fall into chunk c.
__global__ __launch_bounds__(256) void k_apply_ranges(const LayerDev *__restrict__ layers,
                                                      const ChunkInfo *__restrict__ chunk_info,
                                                      uint32_t n_chunks, int n_msgs, const ApplyMsgs msgs,
                                                      uint32_t *__restrict__ ranges) {
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    if (t >= n_chunks * static_cast<uint32_t>(n_msgs)) return;
    const uint32_t k = t / n_chunks, c = t - k * n_chunks;
    const ChunkInfo ci = chunk_info[c];
    const int32_t raw = msgs.counts[k][ci.layer];
    const uint32_t n = static_cast<uint32_t>(min(max(raw, 0), static_cast<int32_t>(min(ci.cap, 0x7fffffffu))));
    const uint32_t *__restrict__ seg = msgs.idx[k] + ci.out_off;
    const uint32_t a = lower_bound_u32(seg, n, ci.start);
    const uint32_t b = ci.last ? n : lower_bound_u32(seg, n, ci.start + ci.len);
    ranges[2 * t] = a;
    ranges[2 * t + 1] = max(a, b);
}

__global__ __launch_bounds__(256) void k_apply_chunks(const ChunkInfo *__restrict__ chunk_info, uint32_t n_chunks,
                                                      int n_msgs, const ApplyMsgs msgs,
                                                      const uint32_t *__restrict__ ranges,
                                                      float *__restrict__ weights, float eta) {
    __shared__ float acc[kChunk];
    __shared__ uint32_t touched[kChunk / 32];
    __shared__ uint32_t s_rng[RSDGC_MAX_MSGS][2];
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const ChunkInfo ci = chunk_info[c];
    uint32_t mine = 0;
    if (tid < n_msgs) {
        const uint32_t a = ranges[2 * (static_cast<uint32_t>(tid) * n_chunks + c)];
        const uint32_t b = ranges[2 * (static_cast<uint32_t>(tid) * n_chunks + c) + 1];
        s_rng[tid][0] = a;
        s_rng[tid][1] = b;
        mine = b - a;
    }
    if (!__syncthreads_or(mine != 0u)) return;         // no message names an element of this chunk
#pragma unroll
    for (int j = 0; j < kChunk / 256; ++j) acc[tid + 256 * j] = 0.f;
    touched[tid] = 0u;
    __syncthreads();
    for (int k = 0; k < n_msgs; ++k) {                 // the sum, message by message, in the order given
        const uint32_t a = s_rng[k][0], b = s_rng[k][1];
        const uint32_t *__restrict__ idx = msgs.idx[k] + ci.out_off;
        const float *__restrict__ val = msgs.val[k] + ci.out_off;
        for (uint32_t j = a + tid; j < b; j += 256) {
            const uint32_t rel = idx[j] - ci.start;
            if (rel < ci.len) {                        // (always, for a sorted message)
                acc[rel] = acc[rel] + val[j];
                atomicOr(&touched[rel >> 5], 1u << (rel & 31));
            }
        }
        __syncthreads();
    }
    uint32_t word = touched[tid];
    float *__restrict__ w = weights + ci.arena_off;
    while (word) {
        const uint32_t rel = 32u * static_cast<uint32_t>(tid) + static_cast<uint32_t>(__ffs(word)) - 1u;
        word &= word - 1u;
        const float sum = acc[rel];
        if (__float_as_uint(sum) != 0u) w[rel] = w[rel] - __fmul_rn(eta, sum);
    }
}

// One message: every pair on its own.
__global__ __launch_bounds__(256) void k_apply_single(const LayerDev *__restrict__ layers, int n_layers,
                                                      long long capacity, const uint32_t *__restrict__ idx,
                                                      const float *__restrict__ val,
                                                      const int32_t *__restrict__ counts,
                                                      float *__restrict__ weights, float eta) {
    const long long j = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
    if (j >= capacity) return;
    int lo = 0, hi = n_layers;            // last layer whose segment starts at or before j
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (layers[mid].out_off <= j) lo = mid; else hi = mid;
    }
    const LayerDev L = layers[lo];
    const long long q = j - L.out_off;
    if (q >= counts[lo] || q >= static_cast<long long>(L.cap)) return;
    const uint32_t i = idx[j];
    if (i >= L.G) return;                 // malformed message: ignore the pair
    const float sum = 0.f + val[j];       // (the sum of one message, formed like any other: +0 + val)
    const size_t pos = static_cast<size_t>(L.elem_off) + i;
    if (__float_as_uint(sum) != 0u) weights[pos] = weights[pos] - __fmul_rn(eta, sum);
}

// Block messages (the block reading): one thread per kept block of every message.  The block
// belongs to the lowest-numbered message that names it (the others find it there by binary
// search in the layer's ascending block list and step aside); its owner looks the block up in
// the later messages, adds their values slot by slot in message order -- plain float32 adds
// starting from +0, as for element messages -- and updates the block's slots inside the matrix.
// No atomics, no scratch memory.
template <int P>
__device__ __forceinline__ void apply_block(const LayerDev &O, int layer, uint32_t b, int k, uint32_t q,
                                            int n_msgs, const ApplyMsgs &msgs,
                                            float *__restrict__ weights, float eta) {
    float sum[P * P];
    {
        const float *__restrict__ src = msgs.val[k] + O.out_off + static_cast<size_t>(q) * (P * P);
#pragma unroll
        for (int s = 0; s < P * P; ++s) sum[s] = 0.f + src[s];
    }
    for (int k2 = k + 1; k2 < n_msgs; ++k2) {
        const uint32_t n2 = static_cast<uint32_t>(min(max(msgs.counts[k2][layer], 0), static_cast<int32_t>(O.k)));
        const uint32_t *__restrict__ seg = msgs.idx[k2] + O.centre_off;
        const uint32_t pos = lower_bound_u32(seg, n2, b);
        if (pos < n2 && seg[pos] == b) {
            const float *__restrict__ src = msgs.val[k2] + O.out_off + static_cast<size_t>(pos) * (P * P);
#pragma unroll
            for (int s = 0; s < P * P; ++s) sum[s] = sum[s] + src[s];
        }
    }
    const int R = static_cast<int>(O.R), C = static_cast<int>(O.C);
    const uint32_t BC = (O.C + P - 1) / P;
    const int bx = static_cast<int>(b / BC), by = static_cast<int>(b - static_cast<uint32_t>(bx) * BC);
#pragma unroll
    for (int dx = 0; dx < P; ++dx)
#pragma unroll
        for (int dy = 0; dy < P; ++dy) {
            const int x = bx * P + dx, y = by * P + dy;
            if (x < R && y < C) {
                const size_t pos = static_cast<size_t>(O.elem_off) + static_cast<size_t>(x) * C + y;
                const float t = sum[dx * P + dy];
                if (__float_as_uint(t) != 0u) weights[pos] = weights[pos] - __fmul_rn(eta, t);
            }
        }
}

__global__ __launch_bounds__(256) void k_apply_blocks(const LayerDev *__restrict__ outer, int n_layers,
                                                      long long capacity, int n_msgs, const ApplyMsgs msgs,
                                                      float *__restrict__ weights, float eta) {
    const long long j = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
    if (j >= capacity) return;
    const int k = blockIdx.y;
    int lo = 0, hi = n_layers;            // last layer whose block segment starts at or before j
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (outer[mid].centre_off <= j) lo = mid; else hi = mid;
    }
    const LayerDev O = outer[lo];
    const long long q = j - O.centre_off;
    if (q >= msgs.counts[k][lo] || q >= static_cast<long long>(O.k)) return;
    const uint32_t BC = (O.C + O.p - 1) / O.p, BR = (O.R + O.p - 1) / O.p;
    const uint32_t b = msgs.idx[k][j];
    if (b >= BR * BC) return;             // malformed message: ignore the block
    for (int k2 = 0; k2 < k; ++k2) {      // an earlier message that names the block owns it
        const uint32_t n2 = static_cast<uint32_t>(min(max(msgs.counts[k2][lo], 0), static_cast<int32_t>(O.k)));
        const uint32_t *__restrict__ seg = msgs.idx[k2] + O.centre_off;
        const uint32_t pos = lower_bound_u32(seg, n2, b);
        if (pos < n2 && seg[pos] == b) return;
    }
    switch (O.p) {
        case 1: apply_block<1>(O, lo, b, k, static_cast<uint32_t>(q), n_msgs, msgs, weights, eta); break;
        case 3: apply_block<3>(O, lo, b, k, static_cast<uint32_t>(q), n_msgs, msgs, weights, eta); break;
        case 5: apply_block<5>(O, lo, b, k, static_cast<uint32_t>(q), n_msgs, msgs, weights, eta); break;
        default: apply_block<7>(O, lo, b, k, static_cast<uint32_t>(q), n_msgs, msgs, weights, eta); break;
    }
}

// ------------------------------------------------------- dynamic ratios --
// Section III-B, Eqs. 3-5: one ranking of mu = |w| over all layers; the K top-ranked weights
// survive and a layer's keep ratio is its share of survivors.  The K-th largest 31-bit key
// (the bit pattern of |w|) is found by a radix select over three streaming passes
// (12 + 10 + 9 bits), a fourth pass counts per layer the keys above and at the threshold.
__global__ __launch_bounds__(256) void k_dyn_init(DynState *__restrict__ state,
                                                  unsigned long long *__restrict__ hist,
                                                  uint32_t *__restrict__ cnt, uint32_t n_cnt,
                                                  unsigned long long K) {
    const int tid = threadIdx.x;
    if (tid == 0) {
        DynState s;
        s.k_rem = K;
        s.prefix = 0;
        s.pad_ = 0;
        *state = s;
    }
    for (int b = tid; b < kHistBins; b += 256) hist[b] = 0ull;
    for (uint32_t i = tid; i < n_cnt; i += 256) cnt[i] = 0u;
}

// Histogram of the digit (key >> shift) & (2^bits - 1) over the keys whose higher bits
// (key >> prev_shift) equal the resolved prefix.  Persistent workgroups stride over the
// 8192-element chunks (padding between layers is never read).
__global__ __launch_bounds__(256) void k_dyn_hist(const ChunkInfo *__restrict__ chunk_info,
                                                  uint32_t n_chunks, const uint32_t *__restrict__ w,
                                                  const DynState *__restrict__ state, int shift,
                                                  int bits, int prev_shift,
                                                  unsigned long long *__restrict__ hist) {
    __shared__ uint32_t lhist[kHistBins];
    const int tid = threadIdx.x;
    const int nb = 1 << bits;
    for (int b = tid; b < nb; b += 256) lhist[b] = 0;
    __syncthreads();
    const uint32_t prefix = state->prefix;
    const uint32_t dmask = static_cast<uint32_t>(nb - 1);
    for (uint32_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const ChunkInfo ci = chunk_info[c];
        const uint32_t *__restrict__ src = w + ci.arena_off;
        for (uint32_t e = 4 * tid; e < ci.len; e += 1024) {
            uint32_t kk[4] = {0, 0, 0, 0};
            uint32_t nv = min(4u, ci.len - e);
            if (nv == 4) {
                typedef uint32_t vu4 __attribute__((ext_vector_type(4)));   // read once per pass: streamed
                const vu4 qq = __builtin_nontemporal_load(reinterpret_cast<const vu4 *>(src + e));
                const uint4 q = make_uint4(qq.x, qq.y, qq.z, qq.w);
                kk[0] = q.x; kk[1] = q.y; kk[2] = q.z; kk[3] = q.w;
            } else {
                for (uint32_t q = 0; q < nv; ++q) kk[q] = src[e + q];
            }
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) {
                const uint32_t key = kk[q] & 0x7fffffffu;
                if (q < nv && (prev_shift >= 31 || (key >> prev_shift) == prefix))
                    atomicAdd(&lhist[(key >> shift) & dmask], 1u);
            }
        }
    }
    __syncthreads();
    for (int b = tid; b < nb; b += 256) {
        const uint32_t c = lhist[b];
        if (c) atomicAdd(&hist[b], static_cast<unsigned long long>(c));
    }
}

// One workgroup: the digit that holds the k_rem-th largest key; clears the histogram.
__global__ __launch_bounds__(256) void k_dyn_find(DynState *__restrict__ state,
                                                  unsigned long long *__restrict__ hist, int bits) {
    __shared__ unsigned long long tot[256];
    const int tid = threadIdx.x;
    const int nb = 1 << bits, per = nb >> 8;   // bits >= 8
    const DynState st = *state;
    const int hi = nb - tid * per;             // thread t owns bins [hi - per, hi): t = 0 holds the top bins
    unsigned long long own = 0;
    for (int b = hi - 1; b >= hi - per; --b) own += hist[b];
    tot[tid] = own;
    __syncthreads();
    if (tid == 0) {                            // 256 partial sums: a serial walk is short enough
        unsigned long long acc = 0;
        int t = 0;
        while (t < 255 && acc + tot[t] < st.k_rem) acc += tot[t++];
        const int h2 = nb - t * per;
        int digit = h2 - per;
        for (int b = h2 - 1; b >= h2 - per; --b) {
            const unsigned long long c = hist[b];
            if (acc + c >= st.k_rem) { digit = b; break; }
            acc += c;
        }
        DynState ns = st;
        ns.prefix = (st.prefix << bits) | static_cast<uint32_t>(digit);
        ns.k_rem = st.k_rem - acc;
        *state = ns;
    }
    __syncthreads();
    for (int b = tid; b < nb; b += 256) hist[b] = 0ull;
}

// Per layer: keys above the threshold and keys equal to it.  Persistent workgroups; the
// counts of a layer are added to its two counters once per workgroup.
__global__ __launch_bounds__(256) void k_dyn_count(const ChunkInfo *__restrict__ chunk_info,
                                                   uint32_t n_chunks, const uint32_t *__restrict__ w,
                                                   const DynState *__restrict__ state,
                                                   uint32_t *__restrict__ cnt /*[n_layers][2]*/) {
    __shared__ uint32_t s_gt, s_eq;
    const int tid = threadIdx.x;
    const uint32_t T = state->prefix;          // all 31 bits are resolved
    if (tid == 0) { s_gt = 0; s_eq = 0; }
    __syncthreads();
    uint32_t cur_l = 0xffffffffu;
    uint32_t gt = 0, eq = 0;                   // this thread's counts for cur_l
    for (uint32_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const ChunkInfo ci = chunk_info[c];
        if (ci.layer != cur_l) {               // uniform
            if (cur_l != 0xffffffffu) {
                if (gt) atomicAdd(&s_gt, gt);
                if (eq) atomicAdd(&s_eq, eq);
                __syncthreads();
                if (tid == 0) {
                    if (s_gt) atomicAdd(&cnt[2 * cur_l], s_gt);
                    if (s_eq) atomicAdd(&cnt[2 * cur_l + 1], s_eq);
                    s_gt = 0; s_eq = 0;
                }
                __syncthreads();
                gt = eq = 0;
            }
            cur_l = ci.layer;
        }
        const uint32_t *__restrict__ src = w + ci.arena_off;
        for (uint32_t e = tid; e < ci.len; e += 256) {
            const uint32_t key = src[e] & 0x7fffffffu;
            gt += key > T ? 1u : 0u;
            eq += key == T ? 1u : 0u;
        }
    }
    if (cur_l != 0xffffffffu) {
        if (gt) atomicAdd(&s_gt, gt);
        if (eq) atomicAdd(&s_eq, eq);
        __syncthreads();
        if (tid == 0) {
            if (s_gt) atomicAdd(&cnt[2 * cur_l], s_gt);
            if (s_eq) atomicAdd(&cnt[2 * cur_l + 1], s_eq);
        }
    }
}

// ------------------------------------------------------------ host side --
int upload_tables(rsdgc_plan_s *plan, void *workspace, hipStream_t stream) {
    if (plan->uploaded_ws == workspace && plan->uploaded_version == plan->version) return RSDGC_OK;
    HIP_TRY(hipMemcpyAsync(workspace, plan->table.data(), plan->ws.table_bytes,
                           hipMemcpyHostToDevice, stream));
    plan->calls_since_upload = 0;
    plan->uploaded_ws = workspace;
    plan->uploaded_version = plan->version;
    return RSDGC_OK;
}

// Workgroups of 256 threads of `kernel` that the whole device keeps resident at once: a
// persistent launch of exactly this many workgroups runs as a single balanced wave.
template <typename K>
uint32_t resident_workgroups(K kernel) {
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 256, 0) != hipSuccess || per_cu < 1)
        per_cu = 2;
    return kNumCUs * static_cast<uint32_t>(per_cu);
}

// One launch of the NSI kernel per neighbourhood side.  kPassSample runs over the sampled
// tiles of the large layers, every other pass over all tiles (workgroups of layers that
// are in another mode leave at once).
struct Momentum {                 // Eq. 12's momentum term; all null / 0 without it
    const float *in = nullptr;
    float *out = nullptr;
    float m = 0.f;
};

template <int PASS>
int launch_nsi(const rsdgc_plan_s *plan, char *ws, const float *grad, const float *resid,
               float *nsi_out, float *v_out, const Momentum &mom, hipStream_t stream,
               bool with_sampled_tiles = true) {
    NsiArgs a;
    a.v_out = v_out;
    a.mom = mom.in;
    a.mom_out = mom.out;
    a.m = mom.m;
    a.flags = reinterpret_cast<const uint32_t *>(ws + plan->ws.flags);
    a.hist_s = reinterpret_cast<uint32_t *>(ws + plan->ws.hist_s);
    a.layers = reinterpret_cast<const LayerDev *>(ws + plan->ws.layers);
    a.grad = grad;
    a.resid = resid;
    a.nsi_out = nsi_out;
    a.hist = reinterpret_cast<uint32_t *>(ws + plan->ws.hist);
    a.state = reinterpret_cast<const SelState *>(ws + plan->ws.state);
    a.state_rw = reinterpret_cast<SelState *>(ws + plan->ws.state);
    a.slot_cnt = reinterpret_cast<uint32_t *>(ws + plan->ws.slot_cnt);
    a.slot_ent = reinterpret_cast<unsigned long long *>(ws + plan->ws.slot_ent);
    a.ca = a.cb = 0.0;                 // set per neighbourhood side below
    const DirEntry *tile_dir = reinterpret_cast<const DirEntry *>(ws + plan->ws.tile_dir);
    const DirEntry *large_dir = reinterpret_cast<const DirEntry *>(ws + plan->ws.large_dir);
    // the main pass and its fallback concern the large layers only: they walk those layers' tiles
    constexpr bool kLargeOnly = PASS == kPassCapture || PASS == kPassFullMap;
    const SampleEntry *samples = reinterpret_cast<const SampleEntry *>(ws + plan->ws.samples);
    uint32_t *feed = reinterpret_cast<uint32_t *>(ws + plan->ws.feed);
    int group_index = 0;
    for (const PGroup &g : plan->groups) {
        // this launch's work-feed counters (cleared at the start of the call)
        const int pass_index = PASS == kPassSample ? 0 : PASS == kPassCapture ? 1 : 2;
        a.feed = feed + static_cast<size_t>((pass_index * 4 + group_index++) % kFeedSets) * kFeedDomains * kFeedStride;
        a.ca = plan->alpha / static_cast<double>(g.p * g.p);
        a.cb = (1.0 - plan->alpha) / static_cast<double>(g.p * g.p);
        a.dir = kLargeOnly ? large_dir + g.large_dir_begin : tile_dir + g.dir_begin;
        a.n_dir = kLargeOnly ? g.large_dir_count : g.dir_count;
        a.n_tiles = g.n_tiles;
        a.samples = samples + g.sample_begin;
        // work items of this launch and the number of workgroups that share them
        // (the first pass without the sampled tiles: only the layers that are always ranked on the full map)
        const uint32_t items = PASS == kPassSample ? (with_sampled_tiles ? g.n_samples : g.n_map_samples)
                                                   : kLargeOnly ? g.n_large_tiles : g.n_tiles;
        if (items == 0) continue;
        a.n_tiles = items;
        a.feed_shift = 7;                  // 128 items per domain and stretch: one per resident workgroup of an XCD
        while (a.feed_shift > 0 && (static_cast<uint32_t>(kFeedDomains) << a.feed_shift) > items) --a.feed_shift;
        const dim3 block(256);
        switch (g.p) {
#define RSDGC_NSI_LAUNCH(PP, MM, FF)                                                        \
    {                                                                                       \
        static const uint32_t resident = resident_workgroups(k_nsi<PP, PASS, MM, FF>);      \
        /* fixed shares: as many workgroups as give every one the same number of tiles    \
           (2786 tiles on 1280 resident workgroups take three rounds either way; 929       \
           workgroups of three tiles each leave the CUs less crowded in all three) */      \
        const uint32_t rounds = (items + resident - 1) / resident;                          \
        const dim3 grid(FF ? std::min<uint32_t>(items, resident) : (items + rounds - 1) / rounds); \
        hipLaunchKernelGGL((k_nsi<PP, PASS, MM, FF>), grid, block, 0, stream, a);           \
    }
#define RSDGC_NSI_CASE(PP)                                                                  \
    case PP: {                                                                              \
        /* the work feed pays when a workgroup gets many tiles (its start and its end cost  \
           a few round trips to the counters); built for the main pass */                   \
        constexpr bool kFeedBuilt = PASS == kPassCapture;                                   \
        const bool fed = kFeedBuilt && plan->work_feed != RSDGC_FEED_OFF &&                 \
                         (plan->work_feed == RSDGC_FEED_ON || items >= 16u * kNumCUs * 4u); \
        if (mom.in) {                                                                       \
            if (fed) RSDGC_NSI_LAUNCH(PP, true, kFeedBuilt)                                 \
            else RSDGC_NSI_LAUNCH(PP, true, false)                                          \
        } else {                                                                            \
            if (fed) RSDGC_NSI_LAUNCH(PP, false, kFeedBuilt)                                \
            else RSDGC_NSI_LAUNCH(PP, false, false)                                         \
        }                                                                                   \
        break;                                                                              \
    }
            RSDGC_NSI_CASE(1)
            RSDGC_NSI_CASE(3)
            RSDGC_NSI_CASE(5)
            RSDGC_NSI_CASE(7)
#undef RSDGC_NSI_CASE
#undef RSDGC_NSI_LAUNCH
            default: return RSDGC_EINVAL;
        }
        HIP_TRY(hipGetLastError());
    }
    return RSDGC_OK;
}

// Records the event that closes `stage` (and opens the next) when profiling is on.
struct StageMarks {
    rsdgc_plan_s *plan;
    hipStream_t stream;
    int base;   // index of this call's first event, -1 when not recording
    StageMarks(rsdgc_plan_s *p, hipStream_t s) : plan(p), stream(s), base(-1) {
        if (!p->prof_events.empty() && p->prof_calls < p->prof_max_calls) {
            base = p->prof_calls * (RSDGC_N_STAGES + 1);
            ++p->prof_calls;
            (void)hipEventRecord(static_cast<hipEvent_t>(p->prof_events[base]), s);
        }
    }
    void close(int stage) {
        if (base >= 0)
            (void)hipEventRecord(static_cast<hipEvent_t>(plan->prof_events[base + stage + 1]), stream);
    }
};

bool aligned256(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

const char *rsdgc_last_hip_error(void) { return g_hip_error; }

// The part of a compress call between the NSI passes and the emit: radix select of every
// layer's threshold, marking of the kept elements, kept counts per chunk and chunk group.
static int select_mark_count(rsdgc_plan_s *plan, char *ws, bool want_centres, StageMarks &marks,
                             PredState *pred, hipStream_t stream) {
    const WsLayout &w = plan->ws;
    const int L = plan->n_layers;
    const uint32_t n_chunks = plan->n_chunks;
    const LayerDev *layers = reinterpret_cast<const LayerDev *>(ws + w.layers);
    const DirEntry *chunk_dir = reinterpret_cast<const DirEntry *>(ws + w.chunk_dir);
    SelState *state = reinterpret_cast<SelState *>(ws + w.state);
    const uint32_t *hist = reinterpret_cast<const uint32_t *>(ws + w.hist);
    uint32_t *flags = reinterpret_cast<uint32_t *>(ws + w.flags);
    uint32_t *chunk_cnt = reinterpret_cast<uint32_t *>(ws + w.chunk_cnt);
    uint32_t *chunk_ccnt = reinterpret_cast<uint32_t *>(ws + w.chunk_ccnt);
    uint32_t *mask = reinterpret_cast<uint32_t *>(ws + w.mask);
    uint32_t *cmask = want_centres ? reinterpret_cast<uint32_t *>(ws + w.cmask) : nullptr;
    float *nsi = reinterpret_cast<float *>(ws + w.nsi);
    const bool inline_count = n_chunks <= kInlineCountChunks;    // small plan: count where the bits are set, no k_count
    const GroupEntry *cand_groups = reinterpret_cast<const GroupEntry *>(ws + w.cand_groups);
    const uint32_t n_cand_groups = static_cast<uint32_t>(plan->cand_groups.size());
    const uint32_t *slot_cnt = reinterpret_cast<const uint32_t *>(ws + w.slot_cnt);
    const unsigned long long *slot_ent = reinterpret_cast<const unsigned long long *>(ws + w.slot_ent);
    // the keys of each layer's threshold bucket are gathered, then one workgroup per layer finishes
    // the ranking on them
    {
        GatherArgs a;
        a.layers = layers;
        a.state = state;
        a.keys = reinterpret_cast<const uint32_t *>(nsi);
        a.slot_cnt = slot_cnt;
        a.slot_ent = slot_ent;
        a.list_cnt = reinterpret_cast<uint32_t *>(ws + w.list_cnt);
        a.list_ent = reinterpret_cast<unsigned long long *>(ws + w.list_ent);
        a.hist = hist;
        a.hist1 = reinterpret_cast<uint32_t *>(ws + w.hist1);
        a.flags = flags;
        a.mask = mask;
        a.cmask = cmask;
        a.chunk_cnt = inline_count ? chunk_cnt : nullptr;
        a.group_cnt = inline_count ? reinterpret_cast<uint32_t *>(ws + w.group_cnt) : nullptr;
        GatherLists gl;
        gl.chunk_dir = chunk_dir;
        gl.map_chunks = reinterpret_cast<const ChunkEntry *>(ws + w.map_chunks);
        gl.cand_groups = cand_groups;
        gl.n_layers = static_cast<uint32_t>(L);
        gl.n_chunks = n_chunks;
        gl.n_map_chunks = static_cast<uint32_t>(plan->map_chunks.size());
        gl.n_cand_groups = n_cand_groups;
        gl.n_map_wgs = std::min<uint32_t>(gl.n_map_chunks, kNumCUs * 4u);
        gl.n_slot_wgs = std::min<uint32_t>(n_cand_groups, kNumCUs * 8u);
        const uint32_t n_fb_wgs = plan->any_large ? std::min<uint32_t>(n_chunks, kNumCUs * 2u) : 0u;
        if (gl.n_map_wgs + gl.n_slot_wgs + n_fb_wgs > 0)
        {
            const dim3 grid(gl.n_map_wgs + gl.n_slot_wgs + n_fb_wgs);
            if (inline_count) hipLaunchKernelGGL(k_gather<true>, grid, dim3(256), 0, stream, a, gl);
            else hipLaunchKernelGGL(k_gather<false>, grid, dim3(256), 0, stream, a, gl);
        }
        uint32_t *list2_cnt = reinterpret_cast<uint32_t *>(ws + w.list2_cnt);
        unsigned long long *list2_ent = reinterpret_cast<unsigned long long *>(ws + w.list2_ent);
        if (plan->big_map_layers)          // long threshold-bucket lists: many workgroups pick the keys k_finish needs
            hipLaunchKernelGGL(k_filter, dim3(L * kFilterSplit), dim3(kFilterThreads), 0, stream, layers, state,
                               a.hist1, a.list_cnt, a.list_ent, list2_cnt, list2_ent);
        hipLaunchKernelGGL(k_finish, dim3(L), dim3(kFinishThreads), 0, stream, layers, state, hist, a.hist1,
                           a.list_cnt, a.list_ent, a.keys, slot_cnt, slot_ent, list2_cnt, list2_ent, pred);
    }
    HIP_TRY(hipGetLastError());
    marks.close(4);

    {
        MarkArgs m;
        m.layers = layers;
        m.state = state;
        m.dir = reinterpret_cast<const DirEntry *>(ws + w.all_tile_dir);
        m.n_layers = static_cast<uint32_t>(L);
        m.n_tiles = plan->n_tiles_all;
        m.map_tiles = reinterpret_cast<const SampleEntry *>(ws + w.map_tiles);
        m.n_map_tiles = static_cast<uint32_t>(plan->map_tiles.size());
        m.n_list_wgs = std::min<uint32_t>(m.n_map_tiles, kNumCUs * 8u);
        m.flags = flags;
        m.keys = reinterpret_cast<const uint32_t *>(nsi);
        m.mask = mask;
        m.cmask = cmask;
        m.chunk_cnt = inline_count ? chunk_cnt : nullptr;
        m.group_cnt = inline_count ? reinterpret_cast<uint32_t *>(ws + w.group_cnt) : nullptr;
        const uint32_t n_fb_wgs = plan->any_large ? std::min<uint32_t>(plan->n_tiles_all, kNumCUs * 4u) : 0u;
        m.n_bucket_wgs = plan->any_large ? static_cast<uint32_t>(L) * kListShards : 0u;
        m.list_cnt = reinterpret_cast<const uint32_t *>(ws + w.list_cnt);
        m.list_ent = reinterpret_cast<const unsigned long long *>(ws + w.list_ent);
        m.slot_cnt = slot_cnt;
        m.slot_ent = slot_ent;
        const uint32_t n_wgs = m.n_bucket_wgs + m.n_list_wgs + n_fb_wgs;
        if (n_wgs > 0) {
            if (inline_count) hipLaunchKernelGGL(k_mark<true>, dim3(n_wgs), dim3(256), 0, stream, m);
            else hipLaunchKernelGGL(k_mark<false>, dim3(n_wgs), dim3(256), 0, stream, m);
        }
    }
    marks.close(5);
    // a small plan's kept elements were counted by the kernels that set their bits; the selected
    // centres, when their lists are wanted, are counted from the centre mask either way
    if (!inline_count || cmask)
        hipLaunchKernelGGL(k_count, dim3(plan->n_count_groups), dim3(kCountThreads), 0, stream,
                           reinterpret_cast<const CountGroup *>(ws + w.count_groups), inline_count ? nullptr : mask,
                           cmask, chunk_cnt, chunk_ccnt, reinterpret_cast<uint32_t *>(ws + w.group_cnt),
                           reinterpret_cast<uint32_t *>(ws + w.group_ccnt),
                           inline_count ? static_cast<uint32_t>(kGroupCntStride) : 1u);
    marks.close(6);
    return RSDGC_OK;
}

static int compress_impl(rsdgc_plan_t *plan, const float *grad, const Momentum &mom,
                         const float *residual, float *residual_out, uint32_t *out_idx,
                         float *out_val, int32_t *out_counts, uint32_t *out_centre_idx,
                         int32_t *out_centre_counts, void *workspace, void *stream_) {
    if (!plan || !grad || !residual || !residual_out || !out_idx || !out_val || !out_counts || !workspace)
        return RSDGC_EINVAL;
    if (plan->blocks) return RSDGC_EINVAL;              // a block plan goes with rsdgc_compress_blocks
    if (!aligned256(workspace) || !aligned16(grad) || !aligned16(residual) || !aligned16(residual_out))
        return RSDGC_EINVAL;
    const bool in_place = residual_out == residual;
    if (!in_place) {    // two arenas: they must not overlap, and the new one must not be the gradient
        const uintptr_t bytes = static_cast<uintptr_t>(plan->total_elems) * sizeof(float);
        const uintptr_t o = reinterpret_cast<uintptr_t>(residual_out);
        const uintptr_t r = reinterpret_cast<uintptr_t>(residual), g = reinterpret_cast<uintptr_t>(grad);
        if ((o < r + bytes && r < o + bytes) || (o < g + bytes && g < o + bytes)) return RSDGC_EINVAL;
    }
    float *v_out = in_place ? nullptr : residual_out;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    char *ws = static_cast<char *>(workspace);
    const WsLayout &w = plan->ws;
    const int L = plan->n_layers;
    const uint32_t n_chunks = plan->n_chunks;
    int rc = upload_tables(plan, workspace, stream);
    if (rc != RSDGC_OK) return rc;
    // the first calls with a workspace (the thresholds have no history yet, or still move fast) may
    // take candidate bounds from a sample of the call's own scores
    const bool sampling = plan->any_large && plan->calls_since_upload < kSamplingCalls;
    if (plan->calls_since_upload < kSamplingCalls) ++plan->calls_since_upload;

    const LayerDev *layers = reinterpret_cast<const LayerDev *>(ws + w.layers);
    SelState *state = reinterpret_cast<SelState *>(ws + w.state);
    uint32_t *hist = reinterpret_cast<uint32_t *>(ws + w.hist);
    uint32_t *flags = reinterpret_cast<uint32_t *>(ws + w.flags);
    PredState *pred = reinterpret_cast<PredState *>(ws + w.pred);
    uint32_t *chunk_cnt = reinterpret_cast<uint32_t *>(ws + w.chunk_cnt);
    uint32_t *chunk_ccnt = reinterpret_cast<uint32_t *>(ws + w.chunk_ccnt);
    const uint32_t *group_cnt = reinterpret_cast<const uint32_t *>(ws + w.group_cnt);
    uint32_t *mask = reinterpret_cast<uint32_t *>(ws + w.mask);
    const bool want_centres = out_centre_idx || out_centre_counts;
    uint32_t *cmask = want_centres ? reinterpret_cast<uint32_t *>(ws + w.cmask) : nullptr;
    float *nsi = reinterpret_cast<float *>(ws + w.nsi);

    StageMarks marks(plan, stream);
    // clear: state .. mask (and the centre mask only when it is used)
    {
        const size_t end = want_centres ? w.zero_end : w.cmask;
        const size_t n16 = (end - w.zero_begin) / 16;
        const unsigned blocks = static_cast<unsigned>(std::min<size_t>((n16 + 255) / 256, 4096));
        hipLaunchKernelGGL(k_begin, dim3(blocks + 1), dim3(256), 0, stream,
                           reinterpret_cast<uint4 *>(ws + w.zero_begin), n16, layers, state, L, pred, flags,
                           sampling ? 1 : 0);
        HIP_TRY(hipGetLastError());
    }
    marks.close(0);

    // first pass: every tile of the layers ranked on the full map (scores, histogram, v) and, where a
    // large layer has no predicted bound, its sampled tiles (histogram only) share one launch.
    // (Running it on a second stream beside the main pass, which does not depend on it once the
    // bounds are predicted, was measured: the two event waits cost more than the overlap gains.)
    rc = launch_nsi<kPassSample>(plan, ws, grad, residual, nsi, v_out, mom, stream, sampling);
    if (rc != RSDGC_OK) return rc;
    if (sampling)
        hipLaunchKernelGGL(k_hint, dim3(L), dim3(256), 0, stream, layers, state,
                           reinterpret_cast<const uint32_t *>(ws + w.hist_s), flags);
    marks.close(1);
    if (plan->any_large) {
        rc = launch_nsi<kPassCapture>(plan, ws, grad, residual, nsi, v_out, mom, stream);
        if (rc != RSDGC_OK) return rc;
    }
    marks.close(2);
    // first ranking digit of every layer, and whether the candidate bounds held
    hipLaunchKernelGGL(k_find0, dim3(L), dim3(256), 0, stream, layers, state, hist, flags, pred);
    if (plan->any_large) {
        // large layers whose candidate bound failed (rare): the workgroups find nothing to do otherwise
        rc = launch_nsi<kPassFullMap>(plan, ws, grad, residual, nsi, v_out, mom, stream);
        if (rc != RSDGC_OK) return rc;
    }
    marks.close(3);

    rc = select_mark_count(plan, ws, want_centres, marks, pred, stream);
    if (rc != RSDGC_OK) return rc;
    const ChunkInfo *chunk_info = reinterpret_cast<const ChunkInfo *>(ws + w.chunk_info);
    if (in_place)
        hipLaunchKernelGGL(k_emit, dim3(n_chunks), dim3(256), 0, stream, layers, chunk_info, grad,
                           residual_out, mask, chunk_cnt, group_cnt, out_idx, out_val, out_counts);
    else
        hipLaunchKernelGGL(k_emit_sparse, dim3(n_chunks), dim3(256), 0, stream, chunk_info, state, grad,
                           residual, residual_out, mom.in, mom.out, mom.m, mask, chunk_cnt, group_cnt, out_idx,
                           out_val, out_counts);
    marks.close(7);
    if (want_centres)                      // the list, the counts, or both
        hipLaunchKernelGGL(k_emit_centres, dim3(n_chunks), dim3(256), 0, stream, layers, chunk_info,
                           cmask, chunk_ccnt, reinterpret_cast<const uint32_t *>(ws + w.group_ccnt), out_centre_idx,
                           out_centre_counts);
    marks.close(8);
    HIP_TRY(hipGetLastError());
    return RSDGC_OK;
}

int rsdgc_compress(rsdgc_plan_t *plan, const float *grad, const float *residual,
                   float *residual_out, uint32_t *out_idx, float *out_val, int32_t *out_counts,
                   uint32_t *out_centre_idx, int32_t *out_centre_counts, void *workspace,
                   void *stream) {
    return compress_impl(plan, grad, Momentum{}, residual, residual_out, out_idx, out_val, out_counts,
                         out_centre_idx, out_centre_counts, workspace, stream);
}

// Workspace of rsdgc_compress_static: one array per GPU, part of the library's code object, so
// that the call needs no device allocation.  It lives as long as the process; every
// rsdgc_compress_static call on a GPU uses that GPU's copy, so two of them must not overlap in
// time on one GPU.  In host code the array's name is not a device address: the address is
// asked for once per device (hipGetSymbolAddress) and only that pointer is handed to kernels
// and copies.
static __device__ __align__(256) unsigned char scratch[RSDGC_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
struct ScratchSlot {
    void *ptr = nullptr;            // device address of `scratch` on this device
    uint64_t owner_serial = 0;      // plan (and its version) whose tables the array holds now
    uint64_t owner_version = 0;
};
ScratchSlot g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;
}  // namespace

int rsdgc_compress_static(rsdgc_plan_t *plan, const float *grad, const float *residual,
                          float *residual_out, uint32_t *out_idx, float *out_val, int32_t *out_counts,
                          uint32_t *out_centre_idx, int32_t *out_centre_counts, void *stream) {
    if (!plan || plan->blocks) return RSDGC_EINVAL;
    if (plan->ws.total > static_cast<size_t>(RSDGC_STATIC_WORKSPACE_BYTES)) {
        std::snprintf(g_hip_error, sizeof(g_hip_error),
                      "rsdgc_compress_static: the plan needs %zu bytes of workspace, the built-in one has %zu",
                      plan->ws.total, static_cast<size_t>(RSDGC_STATIC_WORKSPACE_BYTES));
        return RSDGC_ETOOBIG;
    }
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return RSDGC_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    ScratchSlot &slot = g_scratch[dev];
    if (!slot.ptr) {                       // once per device, with that device current
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || !aligned256(p)) return hip_fail(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
        slot.ptr = p;
    }
    // the array keeps what the last call left: when that was another plan (or other ratios), this
    // plan's tables and its state between calls are laid down again; the per-call clears of
    // rsdgc_compress take care of everything else
    if (slot.owner_serial != plan->serial || slot.owner_version != plan->version) plan->uploaded_ws = nullptr;
    const int rc = compress_impl(plan, grad, Momentum{}, residual, residual_out, out_idx, out_val,
                                 out_counts, out_centre_idx, out_centre_counts, slot.ptr, stream);
    if (rc == RSDGC_OK) {
        slot.owner_serial = plan->serial;
        slot.owner_version = plan->version;
    } else {
        slot.owner_serial = 0;
    }
    return rc;
}

int rsdgc_compress_momentum(rsdgc_plan_t *plan, const float *grad, const float *momentum,
                            float *momentum_out, float m, const float *residual,
                            float *residual_out, uint32_t *out_idx, float *out_val,
                            int32_t *out_counts, uint32_t *out_centre_idx,
                            int32_t *out_centre_counts, void *workspace, void *stream) {
    if (!plan || !grad || !momentum || !momentum_out || !residual || !residual_out) return RSDGC_EINVAL;
    if (!(m >= 0.f && m <= 1.f)) return RSDGC_EINVAL;                       // false for NaN
    if (!aligned16(momentum) || !aligned16(momentum_out)) return RSDGC_EINVAL;
    // five arenas, pairwise disjoint: both new arenas are written while the three inputs are still read
    const uintptr_t bytes = static_cast<uintptr_t>(plan->total_elems) * sizeof(float);
    const uintptr_t p[5] = {reinterpret_cast<uintptr_t>(grad), reinterpret_cast<uintptr_t>(momentum),
                            reinterpret_cast<uintptr_t>(residual), reinterpret_cast<uintptr_t>(momentum_out),
                            reinterpret_cast<uintptr_t>(residual_out)};
    for (int i = 0; i < 5; ++i)
        for (int j = (i < 3 ? 3 : i + 1); j < 5; ++j)
            if (p[i] < p[j] + bytes && p[j] < p[i] + bytes) return RSDGC_EINVAL;
    Momentum mom;
    mom.in = momentum;
    mom.out = momentum_out;
    mom.m = m;
    return compress_impl(plan, grad, mom, residual, residual_out, out_idx, out_val, out_counts,
                         out_centre_idx, out_centre_counts, workspace, stream);
}

// Two arenas of the plan's size overlap unless they are the same one.
static bool arenas_clash(const void *a, const void *b, uintptr_t bytes, bool same_allowed) {
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    if (x == y) return !same_allowed;
    return x < y + bytes && y < x + bytes;
}

static int compress_blocks_impl(rsdgc_plan_t *plan, const float *grad, const Momentum &mom,
                                const float *residual, float *residual_out, uint32_t *out_block_idx,
                                float *out_val, int32_t *out_counts, void *workspace, void *stream_) {
    if (!plan || !plan->blocks || !grad || !residual || !residual_out || !out_block_idx || !out_val ||
        !out_counts || !workspace)
        return RSDGC_EINVAL;
    if (!aligned256(workspace) || !aligned16(grad) || !aligned16(residual) || !aligned16(residual_out))
        return RSDGC_EINVAL;
    {
        // an output arena may be its own input (no element is read by two tiles) and nothing else
        const uintptr_t bytes = static_cast<uintptr_t>(plan->total_elems) * sizeof(float);
        if (arenas_clash(residual_out, residual, bytes, true) || arenas_clash(residual_out, grad, bytes, false))
            return RSDGC_EINVAL;
        if (mom.in) {
            if (!mom.out || !aligned16(mom.in) || !aligned16(mom.out)) return RSDGC_EINVAL;
            if (arenas_clash(mom.out, mom.in, bytes, true) || arenas_clash(mom.out, grad, bytes, false) ||
                arenas_clash(mom.out, residual, bytes, false) || arenas_clash(mom.out, residual_out, bytes, false) ||
                arenas_clash(mom.in, residual_out, bytes, false))
                return RSDGC_EINVAL;
        }
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    char *ws_outer = static_cast<char *>(workspace);
    rsdgc_plan_s *in = plan->inner;
    char *ws = ws_outer + plan->ws.table_bytes;        // the inner plan's workspace
    int rc = upload_tables(plan, workspace, stream);
    if (rc != RSDGC_OK) return rc;
    rc = upload_tables(in, ws, stream);
    if (rc != RSDGC_OK) return rc;
    const WsLayout &w = in->ws;
    const int L = in->n_layers;
    const LayerDev *outer = reinterpret_cast<const LayerDev *>(ws_outer + plan->ws.layers);
    const LayerDev *inner = reinterpret_cast<const LayerDev *>(ws + w.layers);
    const ChunkInfo *inner_chunks = reinterpret_cast<const ChunkInfo *>(ws + w.chunk_info);
    SelState *state = reinterpret_cast<SelState *>(ws + w.state);
    uint32_t *hist = reinterpret_cast<uint32_t *>(ws + w.hist);
    uint32_t *mask = reinterpret_cast<uint32_t *>(ws + w.mask);
    uint32_t *chunk_cnt = reinterpret_cast<uint32_t *>(ws + w.chunk_cnt);
    const uint32_t *group_cnt = reinterpret_cast<const uint32_t *>(ws + w.group_cnt);
    float *score_map = reinterpret_cast<float *>(ws + w.nsi);
    StageMarks marks(in, stream);                      // (the inner plan never records events)
    {
        const size_t n16 = (w.cmask - w.zero_begin) / 16;
        const unsigned blocks = static_cast<unsigned>(std::min<size_t>((n16 + 255) / 256, 4096));
        hipLaunchKernelGGL(k_begin, dim3(blocks + 1), dim3(256), 0, stream,
                           reinterpret_cast<uint4 *>(ws + w.zero_begin), n16, inner, state, L,
                           static_cast<PredState *>(nullptr),    // a block grid is always ranked on its full map
                           reinterpret_cast<uint32_t *>(ws + w.flags), 0);
    }
    bool have[RSDGC_MAX_P + 1] = {};
    for (int l = 0; l < L; ++l) have[plan->p[l]] = true;
    // the work feed (counters in the inner plan's workspace, cleared above) pays when a
    // workgroup gets many tiles
    uint32_t *feed = reinterpret_cast<uint32_t *>(ws + w.feed);
    const bool fed = plan->work_feed != RSDGC_FEED_OFF &&
                     (plan->work_feed == RSDGC_FEED_ON || plan->n_tiles_all >= 16u * kNumCUs * 4u);
    uint32_t feed_shift = 7;
    while (feed_shift > 0 && (static_cast<uint32_t>(kFeedDomains) << feed_shift) > plan->n_tiles_all) --feed_shift;
    for (int pp = 1; pp <= RSDGC_MAX_P; pp += 2) {
        if (!have[pp]) continue;
        switch (pp) {
#define RSDGC_BLOCK_LAUNCH(PP, FF, MM)                                                           \
    {                                                                                            \
        static const uint32_t resident = resident_workgroups(k_block_nsi<PP, FF, MM>);           \
        hipLaunchKernelGGL((k_block_nsi<PP, FF, MM>), dim3(std::min<uint32_t>(plan->n_tiles_all, resident)), \
                           dim3(256), 0, stream, outer,                                          \
                           reinterpret_cast<const DirEntry *>(ws_outer + plan->ws.all_tile_dir), \
                           static_cast<uint32_t>(L), plan->n_tiles_all, inner, grad, residual,   \
                           residual_out, score_map, hist, plan->alpha,                           \
                           feed + static_cast<size_t>(PP / 2) * kFeedDomains * kFeedStride,      \
                           feed_shift, mom.in, mom.out, mom.m);                                  \
    }
#define RSDGC_BLOCK_CASE(PP)                                                                     \
    case PP: {                                                                                   \
        if (mom.in) {                                                                            \
            if (fed) RSDGC_BLOCK_LAUNCH(PP, true, true)                                          \
            else RSDGC_BLOCK_LAUNCH(PP, false, true)                                             \
        } else {                                                                                 \
            if (fed) RSDGC_BLOCK_LAUNCH(PP, true, false)                                         \
            else RSDGC_BLOCK_LAUNCH(PP, false, false)                                            \
        }                                                                                        \
        break;                                                                                   \
    }
            RSDGC_BLOCK_CASE(1)
            RSDGC_BLOCK_CASE(3)
            RSDGC_BLOCK_CASE(5)
            RSDGC_BLOCK_CASE(7)
#undef RSDGC_BLOCK_CASE
#undef RSDGC_BLOCK_LAUNCH
        }
    }
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(k_find0, dim3(L), dim3(256), 0, stream, inner, state, hist,
                       reinterpret_cast<uint32_t *>(ws + w.flags), static_cast<PredState *>(nullptr));
    rc = select_mark_count(in, ws, false, marks, nullptr, stream);
    if (rc != RSDGC_OK) return rc;
    hipLaunchKernelGGL(k_emit_blocks, dim3(in->n_chunks), dim3(256), 0, stream, outer, inner_chunks, mask,
                       chunk_cnt, group_cnt, inner, residual_out, mom.out, out_block_idx, out_val, out_counts);
    HIP_TRY(hipGetLastError());
    return RSDGC_OK;
}

int rsdgc_compress_blocks(rsdgc_plan_t *plan, const float *grad, const float *residual,
                          float *residual_out, uint32_t *out_block_idx, float *out_val,
                          int32_t *out_counts, void *workspace, void *stream) {
    return compress_blocks_impl(plan, grad, Momentum(), residual, residual_out, out_block_idx, out_val,
                                out_counts, workspace, stream);
}

int rsdgc_compress_blocks_momentum(rsdgc_plan_t *plan, const float *grad, const float *momentum,
                                   float *momentum_out, float m, const float *residual,
                                   float *residual_out, uint32_t *out_block_idx, float *out_val,
                                   int32_t *out_counts, void *workspace, void *stream) {
    if (!momentum || !momentum_out || !(m >= 0.f && m <= 1.f)) return RSDGC_EINVAL;
    Momentum mom;
    mom.in = momentum;
    mom.out = momentum_out;
    mom.m = m;
    return compress_blocks_impl(plan, grad, mom, residual, residual_out, out_block_idx, out_val,
                                out_counts, workspace, stream);
}

int rsdgc_decompress_blocks(rsdgc_plan_t *plan, const uint32_t *block_idx, const float *val,
                            const int32_t *counts, float *dense, int accumulate, void *workspace,
                            void *stream_) {
    if (!plan || !plan->blocks || !block_idx || !val || !counts || !dense || !workspace) return RSDGC_EINVAL;
    if (!aligned256(workspace) || !aligned16(dense)) return RSDGC_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    char *ws = static_cast<char *>(workspace);
    int rc = upload_tables(plan, workspace, stream);
    if (rc != RSDGC_OK) return rc;
    const LayerDev *outer = reinterpret_cast<const LayerDev *>(ws + plan->ws.layers);
    if (!accumulate)
        hipLaunchKernelGGL(k_zero_layers, dim3(plan->n_chunks), dim3(256), 0, stream,
                           reinterpret_cast<const ChunkInfo *>(ws + plan->ws.chunk_info), dense);
    if (plan->centre_capacity > 0) {
        const unsigned blocks = static_cast<unsigned>((plan->centre_capacity + 255) / 256);
        hipLaunchKernelGGL(k_scatter_blocks, dim3(blocks), dim3(256), 0, stream, outer, plan->n_layers,
                           static_cast<long long>(plan->centre_capacity), block_idx, val, counts, dense,
                           accumulate);
    }
    HIP_TRY(hipGetLastError());
    return RSDGC_OK;
}

int rsdgc_apply(rsdgc_plan_t *plan, int32_t n_msgs, const uint32_t *const *idx,
                const float *const *val, const int32_t *const *counts, float *weights, float eta,
                void *workspace, void *stream_) {
    if (!plan || plan->blocks || !idx || !val || !counts || !weights || !workspace) return RSDGC_EINVAL;
    if (n_msgs < 1 || n_msgs > RSDGC_MAX_MSGS || !(eta == eta)) return RSDGC_EINVAL;
    if (!aligned256(workspace) || !aligned16(weights)) return RSDGC_EINVAL;
    for (int k = 0; k < n_msgs; ++k)
        if (!idx[k] || !val[k] || !counts[k]) return RSDGC_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    char *ws = static_cast<char *>(workspace);
    int rc = upload_tables(plan, workspace, stream);
    if (rc != RSDGC_OK) return rc;
    const LayerDev *layers = reinterpret_cast<const LayerDev *>(ws + plan->ws.layers);
    if (plan->out_capacity == 0) return RSDGC_OK;      // no message can hold a pair
    if (n_msgs == 1) {
        const unsigned blocks = static_cast<unsigned>((plan->out_capacity + 255) / 256);
        hipLaunchKernelGGL(k_apply_single, dim3(blocks), dim3(256), 0, stream, layers, plan->n_layers,
                           static_cast<long long>(plan->out_capacity), idx[0], val[0], counts[0], weights, eta);
        HIP_TRY(hipGetLastError());
        return RSDGC_OK;
    }
    ApplyMsgs m;
    std::memset(&m, 0, sizeof(m));
    for (int k = 0; k < n_msgs; ++k) {
        m.idx[k] = idx[k];
        m.val[k] = val[k];
        m.counts[k] = counts[k];
    }
    const ChunkInfo *chunk_info = reinterpret_cast<const ChunkInfo *>(ws + plan->ws.chunk_info);
    uint32_t *ranges = reinterpret_cast<uint32_t *>(ws + plan->ws.apply_ranges);
    const uint32_t n_chunks = plan->n_chunks;
    const unsigned range_blocks = static_cast<unsigned>((static_cast<uint64_t>(n_chunks) * n_msgs + 255) / 256);
    hipLaunchKernelGGL(k_apply_ranges, dim3(range_blocks), dim3(256), 0, stream, layers, chunk_info, n_chunks,
                       n_msgs, m, ranges);
    hipLaunchKernelGGL(k_apply_chunks, dim3(n_chunks), dim3(256), 0, stream, chunk_info, n_chunks, n_msgs, m,
                       ranges, weights, eta);
    HIP_TRY(hipGetLastError());
    return RSDGC_OK;
}

int rsdgc_apply_blocks(rsdgc_plan_t *plan, int32_t n_msgs, const uint32_t *const *block_idx,
                       const float *const *val, const int32_t *const *counts, float *weights, float eta,
                       void *workspace, void *stream_) {
    if (!plan || !plan->blocks || !block_idx || !val || !counts || !weights || !workspace) return RSDGC_EINVAL;
    if (n_msgs < 1 || n_msgs > RSDGC_MAX_MSGS || !(eta == eta)) return RSDGC_EINVAL;
    if (!aligned256(workspace) || !aligned16(weights)) return RSDGC_EINVAL;
    for (int k = 0; k < n_msgs; ++k)
        if (!block_idx[k] || !val[k] || !counts[k]) return RSDGC_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    char *ws = static_cast<char *>(workspace);
    int rc = upload_tables(plan, workspace, stream);
    if (rc != RSDGC_OK) return rc;
    const LayerDev *outer = reinterpret_cast<const LayerDev *>(ws + plan->ws.layers);
    if (plan->centre_capacity == 0) return RSDGC_OK;   // no message can hold a block
    const unsigned blocks = static_cast<unsigned>((plan->centre_capacity + 255) / 256);
    ApplyMsgs m;
    std::memset(&m, 0, sizeof(m));
    for (int k = 0; k < n_msgs; ++k) {
        m.idx[k] = block_idx[k];
        m.val[k] = val[k];
        m.counts[k] = counts[k];
    }
    hipLaunchKernelGGL(k_apply_blocks, dim3(blocks, static_cast<unsigned>(n_msgs)), dim3(256), 0, stream, outer,
                       plan->n_layers, static_cast<long long>(plan->centre_capacity), n_msgs, m, weights, eta);
    HIP_TRY(hipGetLastError());
    return RSDGC_OK;
}

int rsdgc_dynamic_ratios(rsdgc_plan_t *plan, const float *weights, double global_ratio,
                         double *ratios_out, void *workspace, void *stream_) {
    if (!plan || plan->blocks || !weights || !ratios_out || !workspace) return RSDGC_EINVAL;
    if (!(global_ratio >= 0.0 && global_ratio <= 1.0)) return RSDGC_EINVAL;     // false for NaN
    if (!aligned256(workspace) || !aligned16(weights)) return RSDGC_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int L = plan->n_layers;
    double n_real = 0.0;
    for (int l = 0; l < L; ++l) n_real += static_cast<double>(plan->layers[l].G);
    double kf = std::ceil(global_ratio * n_real);       // survivors of the ranking (Eq. 4)
    kf = std::min(std::max(kf, 0.0), n_real);
    const unsigned long long K = static_cast<unsigned long long>(kf);
    if (K == 0ull || kf == n_real) {                    // nothing or everything survives
        for (int l = 0; l < L; ++l) ratios_out[l] = K == 0ull ? 0.0 : 1.0;
        return RSDGC_OK;
    }
    char *ws = static_cast<char *>(workspace);
    int rc = upload_tables(plan, workspace, stream);
    if (rc != RSDGC_OK) return rc;
    const WsLayout &w = plan->ws;
    DynState *state = reinterpret_cast<DynState *>(ws + w.dyn);
    unsigned long long *hist = reinterpret_cast<unsigned long long *>(ws + w.dyn + 256);
    uint32_t *cnt = reinterpret_cast<uint32_t *>(ws + w.dyn + 256 + sizeof(unsigned long long) * kHistBins);
    const ChunkInfo *chunk_info = reinterpret_cast<const ChunkInfo *>(ws + w.chunk_info);
    const uint32_t *keys = reinterpret_cast<const uint32_t *>(weights);
    const uint32_t n_chunks = plan->n_chunks;
    const uint32_t grid = std::min<uint32_t>(n_chunks, kNumCUs * 4u);
    hipLaunchKernelGGL(k_dyn_init, dim3(1), dim3(256), 0, stream, state, hist, cnt,
                       static_cast<uint32_t>(2 * L), K);
    int prev_shift = 31;
    for (int lv = 0; lv < 3; ++lv) {                    // 12 + 10 + 9 bits of the 31-bit key
        const int bits = lv == 0 ? 12 : lv == 1 ? 10 : 9, shift = lv == 0 ? 19 : lv == 1 ? 9 : 0;
        hipLaunchKernelGGL(k_dyn_hist, dim3(grid), dim3(256), 0, stream, chunk_info, n_chunks, keys,
                           state, shift, bits, prev_shift, hist);
        hipLaunchKernelGGL(k_dyn_find, dim3(1), dim3(256), 0, stream, state, hist, bits);
        prev_shift = shift;
    }
    hipLaunchKernelGGL(k_dyn_count, dim3(grid), dim3(256), 0, stream, chunk_info, n_chunks, keys, state, cnt);
    HIP_TRY(hipGetLastError());
    std::vector<uint32_t> host;
    try {
        host.resize(2 * static_cast<size_t>(L));
    } catch (const std::bad_alloc &) {
        return RSDGC_ENOMEM;
    }
    HIP_TRY(hipMemcpyAsync(host.data(), cnt, sizeof(uint32_t) * host.size(), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    // survivors per layer: everything above the threshold, then the keys equal to it in layer order
    unsigned long long above = 0, equal = 0;
    for (int l = 0; l < L; ++l) { above += host[2 * l]; equal += host[2 * l + 1]; }
    if (above > K || above + equal < K) {
        std::snprintf(g_hip_error, sizeof(g_hip_error), "rsdgc_dynamic_ratios: inconsistent counts");
        return RSDGC_EHIP;
    }
    unsigned long long remaining = K - above;
    for (int l = 0; l < L; ++l) {
        const unsigned long long take = std::min<unsigned long long>(host[2 * l + 1], remaining);
        remaining -= take;
        ratios_out[l] = static_cast<double>(host[2 * l] + take) / static_cast<double>(plan->layers[l].G);   // Eq. 5
    }
    return RSDGC_OK;
}

int rsdgc_last_paths(rsdgc_plan_t *plan, const void *workspace, int32_t *paths, void *stream_) {
    if (!plan || plan->blocks || !workspace || !paths) return RSDGC_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    std::vector<SelState> host;
    try {
        host.resize(plan->n_layers);
    } catch (const std::bad_alloc &) {
        return RSDGC_ENOMEM;
    }
    HIP_TRY(hipStreamSynchronize(stream));
    HIP_TRY(hipMemcpy(host.data(), static_cast<const char *>(workspace) + plan->ws.state,
                      sizeof(SelState) * plan->n_layers, hipMemcpyDeviceToHost));
    for (int l = 0; l < plan->n_layers; ++l)
        paths[l] = host[l].mode == kModeCandidates && host[l].predicted ? 3 : static_cast<int32_t>(host[l].mode);
    return RSDGC_OK;
}

static void destroy_events(rsdgc_plan_s *plan) {
    for (void *e : plan->prof_events) (void)hipEventDestroy(static_cast<hipEvent_t>(e));
    plan->prof_events.clear();
    plan->prof_max_calls = plan->prof_calls = 0;
}

int rsdgc_profile_begin(rsdgc_plan_t *plan, int32_t max_calls) {
    if (!plan || max_calls < 1 || max_calls > 4096) return RSDGC_EINVAL;
    destroy_events(plan);
    const int n = max_calls * (RSDGC_N_STAGES + 1);
    try {
        plan->prof_events.reserve(n);
    } catch (const std::bad_alloc &) {
        return RSDGC_ENOMEM;
    }
    for (int i = 0; i < n; ++i) {
        hipEvent_t e;
        hipError_t err = hipEventCreate(&e);
        if (err != hipSuccess) {
            destroy_events(plan);
            return hip_fail(err, "hipEventCreate");
        }
        plan->prof_events.push_back(e);
    }
    plan->prof_max_calls = max_calls;
    plan->prof_calls = 0;
    return RSDGC_OK;
}

int rsdgc_profile_end(rsdgc_plan_t *plan, double *stage_ms, int32_t *n_calls) {
    if (!plan || !stage_ms || !n_calls) return RSDGC_EINVAL;
    for (int s = 0; s < RSDGC_N_STAGES; ++s) stage_ms[s] = 0.0;
    *n_calls = plan->prof_calls;
    int rc = RSDGC_OK;
    for (int c = 0; c < plan->prof_calls && rc == RSDGC_OK; ++c) {
        const int base = c * (RSDGC_N_STAGES + 1);
        hipError_t err = hipEventSynchronize(static_cast<hipEvent_t>(plan->prof_events[base + RSDGC_N_STAGES]));
        if (err != hipSuccess) { rc = hip_fail(err, "hipEventSynchronize"); break; }
        for (int s = 0; s < RSDGC_N_STAGES; ++s) {
            float ms = 0.f;
            err = hipEventElapsedTime(&ms, static_cast<hipEvent_t>(plan->prof_events[base + s]),
                                      static_cast<hipEvent_t>(plan->prof_events[base + s + 1]));
            if (err != hipSuccess) { rc = hip_fail(err, "hipEventElapsedTime"); break; }
            stage_ms[s] += ms;
        }
    }
    if (rc == RSDGC_OK && plan->prof_calls > 0)
        for (int s = 0; s < RSDGC_N_STAGES; ++s) stage_ms[s] /= plan->prof_calls;
    destroy_events(plan);
    return rc;
}

const char *rsdgc_stage_name(int32_t stage) {
    static const char *names[RSDGC_N_STAGES] = {"clear", "first_pass", "capture", "find0_fallback", "select",
                                                "mark", "count_scan", "emit", "centres"};
    return (stage >= 0 && stage < RSDGC_N_STAGES) ? names[stage] : "";
}

int rsdgc_nsi(rsdgc_plan_t *plan, const float *grad, const float *residual, float *nsi_out,
              void *workspace, void *stream_) {
    if (!plan || plan->blocks || !grad || !nsi_out || !workspace) return RSDGC_EINVAL;
    if (!aligned256(workspace) || !aligned16(grad) || !aligned16(nsi_out) ||
        (residual && !aligned16(residual)))
        return RSDGC_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = upload_tables(plan, workspace, stream);
    if (rc != RSDGC_OK) return rc;
    return launch_nsi<kPassMapOnly>(plan, static_cast<char *>(workspace), grad, residual, nsi_out,
                                    nullptr, Momentum{}, stream);
}

int rsdgc_decompress(rsdgc_plan_t *plan, const uint32_t *idx, const float *val,
                     const int32_t *counts, float *dense, int accumulate, void *workspace,
                     void *stream_) {
    if (!plan || plan->blocks || !idx || !val || !counts || !dense || !workspace) return RSDGC_EINVAL;
    if (!aligned256(workspace) || !aligned16(dense)) return RSDGC_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    char *ws = static_cast<char *>(workspace);
    int rc = upload_tables(plan, workspace, stream);
    if (rc != RSDGC_OK) return rc;
    const LayerDev *layers = reinterpret_cast<const LayerDev *>(ws + plan->ws.layers);
    if (!accumulate)
        hipLaunchKernelGGL(k_zero_layers, dim3(plan->n_chunks), dim3(256), 0, stream,
                           reinterpret_cast<const ChunkInfo *>(ws + plan->ws.chunk_info), dense);
    if (plan->out_capacity > 0) {
        const unsigned blocks = static_cast<unsigned>((plan->out_capacity + 255) / 256);
        hipLaunchKernelGGL(k_scatter, dim3(blocks), dim3(256), 0, stream, layers, plan->n_layers,
                           static_cast<long long>(plan->out_capacity), idx, val, counts, dense,
                           accumulate);
    }
    HIP_TRY(hipGetLastError());
    return RSDGC_OK;
}

}  // extern "C"
