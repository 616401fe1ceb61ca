/*
 * rsdgc.h -- C ABI of the MI355X (gfx950) RS-DGC local gradient compressor.
 *
 * The library implements the per-iteration, per-node sparsifier Sparse(.) of
 * the paper's Eq. 2: for every layer the gradient, plus the residual carried
 * over from earlier iterations (Eq. 12), is viewed as an R x C matrix
 * (Section III-C), the Neighborhood Statistics Indicator (Eqs. 6-10) is
 * evaluated at every element, the k_l = ceil(G_l / p^2 * rho_l) best-ranked
 * neighbourhoods (Eq. 11, Algorithm 1) are kept whole, and their elements are
 * emitted as compacted (index, value) pairs while the rest stays in the
 * residual.
 *
 * Conventions
 *   - All matrices are float32, row-major, R rows x C columns; for a
 *     convolution weight R = out_ch, C = in_ch * kh * kw.
 *   - "arena": one float32 device array holding all layers back to back; layer
 *     l starts at element rsdgc_layer_offset(plan, l), a multiple of 64.
 *     Padding elements between layers are never read or written.
 *   - Pointers marked [device] must be device memory of the current HIP
 *     device; [host] is ordinary host memory.  The caller owns every buffer;
 *     the library never allocates, frees or synchronises device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All device work is enqueued on it and the call returns without waiting.
 *   - Every function returning int returns RSDGC_OK (0) or a negative
 *     RSDGC_E* code.  Arguments are validated before anything is enqueued, so
 *     on RSDGC_EINVAL no buffer has been touched.  Nothing throws or aborts
 *     across this boundary.
 *   - Non-finite gradient values are not detected, and which neighbourhoods win
 *     next to them is unspecified (the paper does not treat them).  A call on
 *     them is still well formed -- k_l neighbourhoods per layer, ascending
 *     indices, values and residual copied bit for bit, no access out of
 *     bounds -- and leaves nothing behind that changes the result of a later
 *     call.
 *   - A plan may be used by one stream at a time.
 */
#ifndef RSDGC_H
#define RSDGC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RSDGC_OK        0
#define RSDGC_EINVAL   (-1)  /* bad argument (null pointer, shape, p, alpha, ratio) */
#define RSDGC_ENOMEM   (-2)  /* host allocation failed */
#define RSDGC_EHIP     (-3)  /* a HIP call failed; see rsdgc_last_hip_error() */
#define RSDGC_ETOOBIG  (-4)  /* rsdgc_compress_static: the plan needs more workspace than the built-in one */

#define RSDGC_MAX_P     7    /* largest supported neighbourhood side */

typedef struct rsdgc_plan_s rsdgc_plan_t;              /* opaque host object */
typedef struct { int64_t rows, cols; } rsdgc_shape_t;  /* matrix view of one layer */

/* ---------------------------------------------------------------- plan --
 * rsdgc_plan: describe the model once (host only, no HIP call).
 *   shapes      [host] n_layers matrix views; rows, cols >= 1, rows*cols < 2^32.
 *   p           neighbourhood side of Eq. 7, odd, 1..RSDGC_MAX_P, used for
 *               every layer unless p_per_layer != NULL.  Half width (p-1)/2;
 *               window slots outside the matrix count as zeros and the
 *               divisor of Eqs. 9-10 is always p*p.
 *   p_per_layer [host] optional n_layers values overriding p (Section III-C:
 *               p is chosen per kind of layer).
 *   alpha       mixing weight of Eq. 8, in [0, 1].
 *   keep_ratio  [host] n_layers per-layer keep fractions rho_l of Eq. 5, each
 *               in [0, 1] (0.001 keeps one element in a thousand).
 *   out_plan    receives the plan; destroy with rsdgc_plan_destroy.
 * The plan fixes k_l (Eq. 11, evaluated in double as ceil((G_l / p^2) * rho_l),
 * clamped to [0, G_l]), arena offsets, output segment offsets and capacities
 * and the workspace size.                                                   */
int rsdgc_plan(const rsdgc_shape_t *shapes, int32_t n_layers, int32_t p,
               const int32_t *p_per_layer, double alpha,
               const double *keep_ratio, rsdgc_plan_t **out_plan);

/* New per-layer keep ratios (the paper refreshes them once per epoch,
 * Section III-B / Algorithm 1).  Recomputes k_l, output offsets, capacities.
 * The workspace size does not change, but rsdgc_out_capacity and
 * rsdgc_centre_capacity may grow: the caller's out_idx / out_val / out_centre_idx
 * buffers must be re-checked against them before the next rsdgc_compress (the
 * library cannot see their sizes and writes up to the new capacities).      */
int rsdgc_plan_set_ratios(rsdgc_plan_t *plan, const double *keep_ratio);

/* How the per-layer ranking (Algorithm 1) is carried out; the result is the same.
 *   RSDGC_PATH_AUTO      every layer whose keep ratio leaves room for it (8 k_l per 16 x 256
 *                        tile within a tile's 512 candidate entries: up to about 14 % for
 *                        p = 3) records only the centres whose score reaches a bound and
 *                        ranks those.  The bound comes from the thresholds the same layer
 *                        ended on in the two calls before (kept in the workspace), or, in
 *                        the first ten calls with a workspace, from a sample of the
 *                        layer's tiles.  A layer falls back to the full map within the call
 *                        when the bound turns out too high or a tile holds too many such
 *                        centres (default).  The other layers are ranked on the full map,
 *                        and so is a layer whose bound would lie outside 2^-40 .. 2^40
 *                        (scores of the order of 1e-12 or 1e12).
 *   RSDGC_PATH_FULL_MAP  every layer writes its full score map and ranks it with
 *                        histogram passes over all elements.                       */
#define RSDGC_PATH_AUTO      0
#define RSDGC_PATH_FULL_MAP  1
int rsdgc_plan_set_path(rsdgc_plan_t *plan, int32_t path);

/* How the main pass hands its tiles to the workgroups; the result is the same.
 *   RSDGC_FEED_AUTO  from per-XCD work counters when a launch has many tiles per
 *                    workgroup (where it is faster), else a fixed strided share (default).
 *   RSDGC_FEED_OFF   always the fixed share.
 *   RSDGC_FEED_ON    always the counters, also for small launches (meant for tests).
 * Returns RSDGC_EINVAL for a null plan or an unknown mode.                          */
#define RSDGC_FEED_AUTO  0
#define RSDGC_FEED_OFF   1
#define RSDGC_FEED_ON    2
int rsdgc_plan_set_work_feed(rsdgc_plan_t *plan, int32_t mode);

/* A plan remembers the address of the workspace it last prepared (its tables
 * uploaded) and skips that work while the address stays the same.  Call this when the memory at that address has been freed,
 * reused or overwritten in the meantime: the next call with any workspace
 * prepares it afresh.  Host side only; no GPU work.                          */
int rsdgc_plan_forget_workspace(rsdgc_plan_t *plan);

void rsdgc_plan_destroy(rsdgc_plan_t *plan);

/* Host queries; l in [0, n_layers).  Invalid arguments give -1 (0 for size_t). */
int32_t rsdgc_n_layers(const rsdgc_plan_t *plan);
int64_t rsdgc_total_elems(const rsdgc_plan_t *plan);             /* arena length incl. padding */
int64_t rsdgc_layer_offset(const rsdgc_plan_t *plan, int32_t l); /* arena offset of layer l    */
int64_t rsdgc_layer_elems(const rsdgc_plan_t *plan, int32_t l);  /* G_l = rows * cols          */
int64_t rsdgc_layer_k(const rsdgc_plan_t *plan, int32_t l);      /* Eq. 11                      */
int64_t rsdgc_out_offset(const rsdgc_plan_t *plan, int32_t l);   /* start of layer l's pairs    */
int64_t rsdgc_out_capacity(const rsdgc_plan_t *plan);            /* sum_l min(k_l p_l^2, G_l)   */
int64_t rsdgc_centre_offset(const rsdgc_plan_t *plan, int32_t l);/* start of layer l's centres  */
int64_t rsdgc_centre_capacity(const rsdgc_plan_t *plan);         /* sum_l k_l                   */
size_t  rsdgc_workspace_bytes(const rsdgc_plan_t *plan);

/* ------------------------------------------------------------- compress --
 * One iteration of the sparsifier for all layers (Eq. 2's Sparse, Algorithm 1
 * inner loop, Eq. 12 with u = g).
 *   grad      [device, const] float32 arena: this iteration's gradient g.
 *   residual  [device, const] float32 arena: the carried residual r (all
 *             zeros before the first iteration); v = r + g is formed with one
 *             float32 add.
 *   residual_out [device] float32 arena that receives the new residual: +0
 *             where v was emitted, v elsewhere.  Either a second arena that
 *             overlaps neither residual nor grad (the caller swaps the two
 *             pointers between iterations; v is stored while the scores are
 *             computed and only the kept elements are touched afterwards:
 *             12 bytes of HBM traffic per element), or residual_out == residual
 *             for an update in place (one more streaming pass over g and r:
 *             20 bytes per element).  Any other overlap is RSDGC_EINVAL.
 *   out_idx   [device] uint32, rsdgc_out_capacity entries.  Layer l's pairs
 *   out_val   [device] float32, same length.     start at rsdgc_out_offset(l);
 *             idx is the flat row-major index x*C + y inside the layer,
 *             strictly ascending; val is v[idx] bit for bit.  Entries past
 *             out_counts[l] inside a segment are left untouched.
 *   out_counts        [device] int32[n_layers]: pairs emitted per layer
 *                     (k_l <= count <= min(k_l p^2, G_l), or 0 when k_l = 0).
 *   out_centre_idx    [device, nullable] uint32, rsdgc_centre_capacity entries:
 *                     the selected neighbourhood centres of layer l, ascending,
 *                     from rsdgc_centre_offset(l) -- the "neighbourhood index"
 *                     of Section III-C.
 *   out_centre_counts [device, nullable] int32[n_layers]: selected centres per
 *                     layer; always equals k_l.  Either of the two may be given
 *                     without the other.
 *   workspace [device] rsdgc_workspace_bytes bytes, 256-byte aligned.  It is
 *             the plan's device-side state: keep the same buffer, unmodified,
 *             between calls that use this plan (switching to another buffer is
 *             allowed at any time and is detected by its address; after the
 *             buffer's memory was recycled, see rsdgc_plan_forget_workspace).
 *             The first call with a workspace, and the first after
 *             rsdgc_plan_set_ratios, rsdgc_plan_set_path or
 *             rsdgc_plan_forget_workspace, copies the plan's tables from host
 *             memory into it (one hipMemcpyAsync on `stream`): that call must
 *             not be made under HIP graph capture; every later one enqueues
 *             kernels only and may be captured.
 * Ranking ties are resolved towards the lower flat index; exactly k_l centres
 * are selected.  Scores are float32 roundings of double-precision window
 * statistics.                                                               */
int rsdgc_compress(rsdgc_plan_t *plan, const float *grad, const float *residual,
                   float *residual_out, uint32_t *out_idx, float *out_val, int32_t *out_counts,
                   uint32_t *out_centre_idx, int32_t *out_centre_counts,
                   void *workspace, void *stream);

/* rsdgc_compress for callers that cannot allocate device memory (code that runs under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * workspace is an array inside the library, RSDGC_STATIC_WORKSPACE_BYTES long, one copy
 * per GPU, held from the moment the library is loaded until the process ends.  The call
 * allocates and frees nothing, on the device or through any library that would.
 *   - Arguments and results as for rsdgc_compress (same kernels), without `workspace`.
 *     The caller still owns inputs and outputs.
 *   - A plan with rsdgc_workspace_bytes(plan) > RSDGC_STATIC_WORKSPACE_BYTES is refused
 *     with RSDGC_ETOOBIG before anything is enqueued (rsdgc_last_hip_error() then holds
 *     both sizes); a block plan with RSDGC_EINVAL.
 *   - All calls on one GPU share that GPU's array: two of them (from any plans, streams
 *     or threads) must not overlap in time -- the later one would overwrite tables and
 *     counters the earlier one still reads.  Calls that follow each other on one stream
 *     are fine.  When the array last served another plan (or this plan with other ratios),
 *     the plan's tables are copied into it again (one host-to-device copy on `stream`)
 *     and a state the plan keeps between calls starts afresh; everything else that must
 *     start at zero is cleared by every call.
 *   - The device current at the time of the call is the one whose array is used.      */
#define RSDGC_STATIC_WORKSPACE_BYTES (64u << 20)
int rsdgc_compress_static(rsdgc_plan_t *plan, const float *grad, const float *residual,
                          float *residual_out, uint32_t *out_idx, float *out_val,
                          int32_t *out_counts, uint32_t *out_centre_idx,
                          int32_t *out_centre_counts, void *stream);

/* The same iteration with momentum correction (Eq. 12 in full; Section III-C's last
 * paragraph adopts it):  u = m*u + g  (one float32 multiply, one float32 add),
 * v = r + u, then everything as in rsdgc_compress on that v.  Where v was
 * emitted the momentum restarts from +0 together with the residual (the masking
 * of the method Eq. 12 is taken from).
 *   momentum      [device, const] float32 arena: u of the previous iteration
 *                 (all zeros before the first).
 *   momentum_out  [device] float32 arena that receives the new u.
 *   m             momentum factor in [0, 1]; m = 0 gives rsdgc_compress's result.
 * grad, momentum, residual, momentum_out and residual_out must be five arenas that
 * do not overlap (there is no in-place form); anything else is RSDGC_EINVAL.
 * All other arguments as for rsdgc_compress.  HBM traffic: 20 bytes per element.  */
int rsdgc_compress_momentum(rsdgc_plan_t *plan, const float *grad, const float *momentum,
                            float *momentum_out, float m, const float *residual,
                            float *residual_out, uint32_t *out_idx, float *out_val,
                            int32_t *out_counts, uint32_t *out_centre_idx,
                            int32_t *out_centre_counts, void *workspace, void *stream);

/* Dynamic compression strategy (Section III-B, Eqs. 3-5; Algorithm 1's per-epoch part):
 * mu = |w| of every weight of the network is ranked across all layers, the
 * ceil(global_ratio * G) top-ranked weights survive (equal |w|: earlier layer
 * first), and layer l's keep ratio is survivors_l / G_l.
 *   weights     [device, const] float32 arena laid out like the gradient arena.
 *   ratios_out  [host] double[n_layers]; feed it to rsdgc_plan_set_ratios.
 * Runs four streaming passes on `stream` and waits for them (a per-epoch step,
 * not part of the per-iteration path); uses the workspace's scratch only, so it
 * must not overlap a compress call that uses the same workspace.             */
int rsdgc_dynamic_ratios(rsdgc_plan_t *plan, const float *weights, double global_ratio,
                         double *ratios_out, void *workspace, void *stream);

/* NSI map only (Eqs. 8-10 at every element of every layer), for inspection:
 *   residual [device, nullable] NULL means an all-zero residual.
 *   nsi_out  [device] float32 arena; padding elements are not written.
 * Neither grad nor residual is modified.                                    */
int rsdgc_nsi(rsdgc_plan_t *plan, const float *grad, const float *residual,
              float *nsi_out, void *workspace, void *stream);

/* ----------------------------------------------------------- decompress --
 * Scatter one message back into a dense arena (the sum over nodes of
 * sparse(v) in Eq. 12's third line is formed by calling this once per
 * message with accumulate = 1).
 *   idx, val, counts  [device] as produced by rsdgc_compress with this plan.
 *   dense             [device] float32 arena.
 *   accumulate = 0: every layer element of dense is overwritten (zeros where
 *                   nothing was sent);  != 0: dense[idx] += val.
 * A message is taken as it comes (it may have crossed a network): a pair
 * whose index is not below G_l is skipped, counts[l] is read as clamped to
 * [0, the layer's segment capacity], and nothing outside dense's layer
 * elements is ever written; none of this is reported as an error.  A message
 * that names an element twice (rsdgc_compress never does) leaves an
 * unspecified one of its values, or sums, there.  The same holds for
 * rsdgc_decompress_blocks (block index not below the layer's block count) and
 * for the messages given to rsdgc_apply and rsdgc_apply_blocks.             */
int rsdgc_decompress(rsdgc_plan_t *plan, const uint32_t *idx, const float *val,
                     const int32_t *counts, float *dense, int accumulate,
                     void *workspace, void *stream);

/* ---------------------------------------------------------- block reading --
 * The other reading of Section III-C ("a convolution kernel as a whole", the
 * G / p^2 of Eq. 11): the matrix is cut into ceil(R/p) x ceil(C/p)
 * non-overlapping p x p blocks and each block is one neighbourhood.  Its NSI is
 * Eqs. 8-10 over the block's p*p slots (zero outside the matrix, divisor p*p);
 * the k_l = ceil(G_l / p^2 * rho_l) best blocks are kept (ties: lower block
 * index) and a kept block goes out as its index plus its p*p values.
 *
 * rsdgc_plan_blocks has rsdgc_plan's arguments.  For such a plan
 *   rsdgc_layer_k(l)            kept blocks of layer l,
 *   rsdgc_centre_offset(l) / rsdgc_centre_capacity   layout of the block index list,
 *   rsdgc_out_offset(l) / rsdgc_out_capacity         layout of the value list
 *                               (k_l * p_l^2 floats per layer),
 * and only rsdgc_compress_blocks(_momentum) / rsdgc_decompress_blocks / rsdgc_apply_blocks (and
 * the plan calls) accept it; a plan from rsdgc_plan is refused by these (RSDGC_EINVAL).
 *   out_block_idx [device] uint32: per layer, from rsdgc_centre_offset(l), the kept
 *                 blocks' indices bx * ceil(C/p) + by, ascending.
 *   out_val       [device] float32: per layer, from rsdgc_out_offset(l), p*p values
 *                 per kept block in the same order, row-major inside the block,
 *                 +0 for slots outside the matrix.
 *   out_counts    [device] int32[n_layers]: kept blocks per layer (= k_l).
 *   residual_out  a second arena, or residual itself (blocks share no element, so
 *                 the update in place costs nothing extra here).
 * Everything else as for rsdgc_compress / rsdgc_decompress.                  */
int rsdgc_plan_blocks(const rsdgc_shape_t *shapes, int32_t n_layers, int32_t p,
                      const int32_t *p_per_layer, double alpha,
                      const double *keep_ratio, rsdgc_plan_t **out_plan);
int rsdgc_compress_blocks(rsdgc_plan_t *plan, const float *grad, const float *residual,
                          float *residual_out, uint32_t *out_block_idx, float *out_val,
                          int32_t *out_counts, void *workspace, void *stream);
/* The block reading with momentum correction (Eq. 12 in full, Section III-C's last paragraph):
 * u = m*u + g (one float32 multiply, one float32 add), v = r + u, then the blocks are scored,
 * ranked and sent as in rsdgc_compress_blocks on that v; momentum and residual both restart
 * from +0 on every slot of a kept block.
 *   momentum      [device, const] float32 arena: u of the previous iteration.
 *   momentum_out  [device] float32 arena for the new u: a further arena, or momentum itself.
 *   m             momentum factor in [0, 1]; m = 0 gives rsdgc_compress_blocks's message.
 * Apart from momentum_out == momentum and residual_out == residual no two arenas may overlap
 * (RSDGC_EINVAL).  HBM traffic: 20 bytes per element.                                        */
int rsdgc_compress_blocks_momentum(rsdgc_plan_t *plan, const float *grad, const float *momentum,
                                   float *momentum_out, float m, const float *residual,
                                   float *residual_out, uint32_t *out_block_idx, float *out_val,
                                   int32_t *out_counts, void *workspace, void *stream);
int rsdgc_decompress_blocks(rsdgc_plan_t *plan, const uint32_t *block_idx, const float *val,
                            const int32_t *counts, float *dense, int accumulate,
                            void *workspace, void *stream);

/* The receiving side of an iteration (Eq. 12, third line):
 *   w <- w - eta * sum_k sparse(v_k)
 * for the messages of n_msgs nodes, each as produced by rsdgc_compress with a
 * plan of the same shapes and ratios.  The messages are summed in the order
 * given (float32 adds, starting from +0), the step is one float32 multiply and
 * one float32 subtract; weights at positions no message names, or whose sum is
 * +0, are not touched.  Only the named positions are visited: the cost is
 * proportional to the messages, not to the model, and no dense accumulator is
 * kept.
 *   idx, val, counts  [host] arrays of n_msgs device pointers (1 <= n_msgs <=
 *                     RSDGC_MAX_MSGS); message k is idx[k], val[k], counts[k].
 *   weights           [device, in/out] float32 arena laid out like the gradient.
 * With more than one message every layer's indices must be ascending, as
 * rsdgc_compress writes them (the pairs of one stretch of a layer are found by
 * binary search); a segment that is not leaves an unspecified part of the sum at
 * its positions, but nothing outside the layers' elements is ever written.  A
 * single message is applied pair by pair, in any order.  Uses scratch inside the
 * workspace: must not overlap another call that uses the same workspace.       */
#define RSDGC_MAX_MSGS 64
int rsdgc_apply(rsdgc_plan_t *plan, int32_t n_msgs, const uint32_t *const *idx,
                const float *const *val, const int32_t *const *counts, float *weights,
                float eta, void *workspace, void *stream);

/* The same for a plan from rsdgc_plan_blocks and messages as produced by
 * rsdgc_compress_blocks: block_idx[k], val[k] (p*p values per block) and
 * counts[k] of node k.  Every layer's block indices must be ascending, as
 * rsdgc_compress_blocks writes them: a block is applied once, by the first
 * message that names it, which finds it in the later ones by binary search.
 * One launch, no scratch memory.  rsdgc_apply refuses a block plan and this
 * call an element plan (RSDGC_EINVAL).                                        */
int rsdgc_apply_blocks(rsdgc_plan_t *plan, int32_t n_msgs, const uint32_t *const *block_idx,
                       const float *const *val, const int32_t *const *counts, float *weights,
                       float eta, void *workspace, void *stream);

/* ------------------------------------------------------------ profiling --
 * Per-stage GPU time of rsdgc_compress, measured with HIP events recorded on the
 * caller's stream between the stages.  rsdgc_profile_begin creates the events for up
 * to max_calls calls (further calls are not recorded); rsdgc_profile_end waits for the
 * recorded events, writes the mean milliseconds per call of each stage into
 * stage_ms[RSDGC_N_STAGES] [host], the number of recorded calls into *n_calls [host],
 * and destroys the events.  Stages: see rsdgc_stage_name.                        */
#define RSDGC_N_STAGES 9
int rsdgc_profile_begin(rsdgc_plan_t *plan, int32_t max_calls);
int rsdgc_profile_end(rsdgc_plan_t *plan, double *stage_ms, int32_t *n_calls);
const char *rsdgc_stage_name(int32_t stage);

/* Which ranking path each layer took in the last rsdgc_compress that used `workspace`:
 * paths[l] [host, n_layers] = 0 candidates above a bound taken from a sample of the layer,
 * 1 full score map, 2 nothing to select (k_l = 0), 3 candidates above a bound predicted
 * from the layer's earlier thresholds.  Waits for `stream`, then copies from the device.
 * The path never changes a result.  A layer that would take path 0 or 3 shows 1 when
 *   - its bound failed in this call (too few centres above it, or too many in one tile):
 *     the call then ranked the full map, and the safety margin of the layer's predicted
 *     bounds is doubled (too few above) or halved, down to its start value (too many); during
 *     the first ten calls with a workspace the next four bounds are sampled ones; later
 *     the next bound is set below this call's threshold, without a trend;
 *   - the workspace is past those ten calls, the only ones that sample tiles, and one
 *     of the layer's last two thresholds is zero or subnormal (nothing to predict from). */
int rsdgc_last_paths(rsdgc_plan_t *plan, const void *workspace, int32_t *paths, void *stream);

/* ----------------------------------------------------------- diagnostics */
const char *rsdgc_strerror(int code);
/* Text of the last HIP error seen by this thread inside the library ("" if none). */
const char *rsdgc_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RSDGC_H */
