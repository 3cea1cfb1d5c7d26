/*
 * osp.h - C ABI of the MI355X-native OSP synchronization step.
 *
 * OSP (Overlapped Synchronization Parallel) splits the per-iteration gradient
 * synchronization of parameter-server training into two stages (Sec. 3.1):
 * the important gradients G^i are synchronized right after back-propagation
 * (Routine Synchronization, RS, "stage 1" here); the unimportant gradients
 * G^u are synchronized while the next iteration computes (In-Computation
 * Synchronization, ICS, "stage 2").  This library is the arithmetic of that
 * step for N workers whose buffers all live on ONE GPU: no transport.
 *
 * Memory model
 *   Every buffer is a flat fp32 "arena" of arena_elems elements; tensor
 *   ("layer") l occupies [offset[l], offset[l]+numel[l]).  Elements outside
 *   every tensor are padding and are never written by any call.  Offsets need
 *   to be multiples of 4 elements only; multiples of 1024 (4 KiB) measure 1.5-2 %
 *   faster per step on MI355X than multiples of 64.
 *   All pointers in osp_buffers and every `grads` argument are DEVICE
 *   pointers owned by the caller and only borrowed: the library never
 *   allocates or frees device memory (osp_bind allocates a few bytes of
 *   pinned host memory, freed by osp_destroy).  Every call of a context is
 *   made with the device current that owns these buffers.  All pointers in osp_config and the
 *   gib/out arguments of osp_set_gib / osp_get_* are HOST pointers.
 *   `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   Kernels are enqueued on it and the call returns without waiting for the
 *   GPU.  That holds for every call of the synchronization step (the staged
 *   calls, the windows, osp_split): launches over a stage of a layer-granular
 *   GIB read the size of the stage on the device, so whole iterations can be
 *   enqueued while an earlier split has not run yet, and a step can be
 *   captured into a HIP graph and replayed.  The calls that do wait: osp_bind,
 *   osp_set_gib and the osp_get_* calls synchronize the stream; osp_n_stage2,
 *   osp_split_gradients and osp_ps_aggregate_update_packed need the stage-2
 *   size on the HOST and wait for a layer-granular split that is still running.
 *   The kernels that read all N gradient arenas at once (the aggregate, LGP
 *   that keeps the stage-2 aggregate, the element-granular windows) are
 *   launched with up to 40 KB of dynamic LDS per one-wavefront workgroup that
 *   they never touch: it bounds how many of them a compute unit holds (fewer
 *   bytes in flight move faster), and it is not available to other kernels on
 *   that compute unit meanwhile.  Gradient arenas that are a multiple of 1 MiB
 *   plus 4 to 32 KiB apart (worker_stride) measure 1-3 % faster in these
 *   kernels than arenas 4 KiB + 768 B apart, and replicas a multiple of 1 KiB
 *   apart (param_stride; say a multiple of 1 MiB plus 1 KiB) 1-3 % faster than
 *   replicas that are not.
 *
 * Concurrency
 *   The calls of one context update shared buffers and must not overlap in
 *   time with each other: enqueue them on one stream, or order the streams
 *   with events.  What OSP overlaps is the stage-2 calls of iteration t with
 *   the COMPUTE of iteration t+1 (Sec. 3.1), which runs on the caller's other
 *   streams and does not touch these buffers' stage-2 elements.  Different
 *   contexts are independent.
 *
 * Errors
 *   Every call returns a status and never throws or aborts.  Argument and
 *   ordering errors are detected on the host before anything is enqueued and
 *   leave all buffers untouched.  osp_last_error gives a message.
 *
 * Order of calls in one iteration (Sec. 3.1, Sec. 4.1.2 Eq. 5, Sec. 4.5)
 *   osp_ps_aggregate_update(1) -> { osp_apply_stage(1), osp_lgp_correct } ->
 *   osp_ps_aggregate_update(2) -> osp_apply_stage(2) -> osp_split
 *   A GIB must exist before any staged call (osp_set_gib with all layers
 *   important makes iteration 1 a plain BSP step, Algorithm 1: S(G^u)_1 = 0).
 *   Violations return OSP_ERR_BAD_STATE:
 *     - stage 2 (aggregate or apply) before stage 1 of the same iteration;
 *     - a new stage 1, stage 0 or osp_set_gib while a stage 2 is pending
 *       (the ICS of iteration t must finish inside iteration t+1's compute
 *       window, Eq. 5);
 *     - osp_lgp_correct twice, or after osp_apply_stage(2);
 *     - osp_split before the iteration's stage 2 (or stage 0) aggregate.
 *   osp_split closes the iteration; calling it is optional (the old GIB stays).
 */
#ifndef OSP_H
#define OSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct osp_ctx osp_ctx;            /* opaque, host memory, library-owned */

typedef enum {
    OSP_OK = 0,
    OSP_ERR_INVALID_ARG = 1,
    OSP_ERR_BAD_STATE = 2,
    OSP_ERR_NOMEM = 3,
    OSP_ERR_HIP = 4,
    OSP_ERR_UNSUPPORTED = 5
} osp_status;

/* Granularity of the Gradient Importance Bitmap (GIB, Sec. 3.2).
 * LAYER is the paper's choice (Eq. 4): one flag per tensor.
 * ELEMENT uses the per-parameter importance I_k = |G_k P_k| (text after Eq. 3). */
enum { OSP_GRAN_LAYER = 0, OSP_GRAN_ELEMENT = 1 };

typedef struct {
    int32_t n_workers;             /* N >= 1 */
    int32_t n_tensors;             /* L >= 1 */
    const int64_t *numel;          /* [L], each > 0; copied */
    const int64_t *offset;         /* [L], ascending, multiples of 4, ranges disjoint; copied */
    int64_t arena_elems;           /* multiple of 4, >= offset[L-1] + numel[L-1] */
    float lr;                      /* learning rate (Sec. 5.1.3: 0.1) */
    float momentum;                /* SGD momentum mu, 0 <= mu < 1 */
    const float *worker_weight;    /* [N] data share alpha_w of each worker (Sec. 2.1.1), or
                                      NULL for equal shares 1/N; copied */
    int32_t element_keys;          /* nonzero: osp_ps_aggregate_update also stores every
                                      element's importance key, which makes
                                      osp_split(OSP_GRAN_ELEMENT) legal (costs 4 B/element of
                                      workspace for the keys, on top of the 4 B/element of
                                      the kept stage-2 aggregate) */
    int32_t chunk_elems;           /* work-chunk size in elements, multiple of 256;
                                      0 = library default (256: one float4 per lane) */
} osp_config;

typedef struct {
    float *ps_param;               /* [arena_elems] global parameters P on the PS */
    float *ps_momentum;            /* [arena_elems] momentum buffer V on the PS */
    float *worker_param;           /* worker w's replica starts at worker_param + w*stride */
    int64_t worker_param_stride;   /* elements, multiple of 4, >= arena_elems */
    void *workspace;               /* 256-byte aligned scratch, >= osp_workspace_bytes();
                                      4 KiB alignment lets its arena-sized arrays start on
                                      4 KiB boundaries like the arenas' tensors */
    size_t workspace_bytes;
    int32_t replicas_in_sync;      /* nonzero: the caller asserts that every replica equals
                                      ps_param on every tensor element right now.  Lets the
                                      first iteration's LGP read the PS values once instead of
                                      N replica values; from the second iteration on the
                                      library knows by itself.  While bound, replicas must be
                                      written through this library only. */
} osp_buffers;

/* Create / destroy a context (host only; no GPU needed). *out is NULL on error. */
osp_status osp_create(const osp_config *cfg, osp_ctx **out);
void osp_destroy(osp_ctx *ctx);                                   /* NULL is fine */

/* Bytes of device workspace osp_bind needs (chunk table, per-chunk importance
 * partials, GIB, and with element_keys the key array, bitmap and histograms). */
size_t osp_workspace_bytes(const osp_ctx *ctx);

/* Attach device buffers; uploads the chunk table into the workspace and clears
 * the GIB state (no GIB afterwards).  All pointers must be 16-byte aligned. */
osp_status osp_bind(osp_ctx *ctx, const osp_buffers *buf, void *stream);

/* Change lr / momentum between iterations (Sec. 5.1.3: lr is halved every 10 epochs). */
osp_status osp_set_hyper(osp_ctx *ctx, float lr, float momentum);

/*
 * Gradient split (Sec. 3.2 first challenge, Sec. 4.1.1, 4.1.2): computes the GIB
 * of the NEXT iteration from this iteration's importances, which
 * osp_ps_aggregate_update accumulated from the aggregated gradient and the PS
 * parameters as they were before the update.
 *   LAYER:   layers are ranked by (I^l, l) ascending, I^l = sum_{k in l}|g_k P_k|
 *            (Eq. 4, summed in fp64); stage 2 = the longest prefix of the ranking
 *            whose element count stays <= budget_elems.
 *   ELEMENT: stage 2 = the budget_elems elements that come first in the order
 *            (I_k ascending, arena index ascending); needs cfg.element_keys.
 * 0 <= budget_elems <= number of parameters, else OSP_ERR_INVALID_ARG.
 * NaN importances rank above +Inf (they stay in stage 1).
 */
osp_status osp_split(osp_ctx *ctx, int granularity, int64_t budget_elems, void *stream);

/*
 * osp_split(OSP_GRAN_ELEMENT) for callers that cannot allocate device memory and
 * have no bound workspace at hand: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Stateless: no context.  Selects the
 * budget_elems smallest of n_elems importance keys in the order (key ascending,
 * index ascending) and writes the element bitmap (bit k%32 of word k/32, 0 =
 * stage 2; [ceil(n_elems/32)] words, bits beyond n_elems come out 1).
 *   keys:        DEVICE, 16-byte aligned, [n_elems]; importance keys as
 *                osp_get_keys returns them (elements that must never be selected,
 *                such as padding, carry 0xFFFFFFFF; budget_elems must not exceed
 *                the number of other keys).  Read-only.
 *   elem_bitmap: DEVICE, 4-byte aligned, caller-owned, overwritten.
 *   n_elems:     positive multiple of 4, at most 2^28 (OSP_ERR_UNSUPPORTED above).
 * The histograms, counters, tie candidates and per-tile counts live in an array
 * of 1.2 MB that is part of the library's image on every GPU it runs on (held
 * until the process ends); the call clears what must start at zero with a fill
 * kernel, launches the kernels osp_split launches, and calls no allocating
 * routine.  Every call on one GPU uses that GPU's one array: calls that overlap
 * in time on one GPU (two streams, two threads) race; order them.  Enqueues on
 * `stream` and returns without waiting; errors as everywhere (message through
 * osp_last_error(NULL)).
 */
osp_status osp_split_element_static(const uint32_t *keys, int64_t n_elems, int64_t budget_elems,
                                    uint32_t *elem_bitmap, void *stream);

/* Read the current GIB back (synchronizes `stream`).  Any of the three outputs
 * may be NULL.  layer_gib: [L] bytes, 1 = important (stage 1), 0 = stage 2;
 * only written when the current GIB is layer-granular.  elem_bitmap:
 * [ceil(arena_elems/32)] words, bit k%32 of word k/32, 1 = important, padding
 * bits 1; only written when it is element-granular.  n_stage2: elements in
 * stage 2.  OSP_ERR_BAD_STATE if there is no GIB. */
osp_status osp_get_gib(osp_ctx *ctx, uint8_t *layer_gib, uint32_t *elem_bitmap,
                       int64_t *n_stage2, void *stream);

/* Enqueue a copy of the current stage-2 element count into *out_host without
 * waiting; out_host should be pinned host memory and is valid once `stream` has
 * passed this point.  For callers that log the split size every iteration
 * without stalling the stream. */
osp_status osp_read_n_stage2_async(osp_ctx *ctx, int64_t *out_host, void *stream);

/* A log of stage-2 sizes without any stream operation per iteration: from now on
 * every osp_split (the one inside osp_ics_window too) also stores the size of the
 * stage 2 it has just chosen at log[k % capacity], k = 0, 1, ... counting the
 * splits since this call.  log: memory the DEVICE can write, 8-byte aligned
 * (device memory, or the device address of mapped pinned host memory),
 * caller-owned, valid until the log is taken away (log = NULL), the context is
 * rebound or destroyed.  Enqueues one small kernel on `stream`; entries are
 * valid once the stream has passed the split that writes them.  Replays of a
 * captured split keep counting. */
osp_status osp_set_stage2_log(osp_ctx *ctx, int64_t *log, int64_t capacity, void *stream);

/* The current stage-2 element count, on the host, without a stream operation:
 * the split publishes it in pinned host memory.  Waits if a layer-granular
 * osp_split is still running (or has not started: do not call it between the
 * capture of a graph that holds a split and the graph's first replay).  Callers
 * that must not wait use osp_read_n_stage2_async. */
osp_status osp_n_stage2(osp_ctx *ctx, int64_t *n_stage2);

/* Install a GIB from the host (first iteration, tests, resume).  gib_host is
 * uint8[L] for LAYER or uint32[ceil(arena_elems/32)] for ELEMENT, same encoding
 * as osp_get_gib; padding bits are ignored.  Synchronizes `stream`. */
osp_status osp_set_gib(osp_ctx *ctx, int granularity, const void *gib_host, void *stream);

/*
 * Parameter-server side of one stage (Sec. 2.1.1, per stage as in Sec. 3.1).
 * For every element k of the stage (1 = important set, 2 = unimportant set,
 * 0 = all elements, i.e. a plain BSP step, Sec. 4.3):
 *     gbar = sum_w alpha_w g_{w,k}      fp32, workers in ascending order;
 *                                       with equal shares: (sum_w g_{w,k}) * fl(1/N)
 *     I_k  = |gbar * P_k|               PGP importance, P before this update
 *     V_k  = mu V_k + gbar ;  P_k = P_k - lr V_k
 * Every operation is a separately rounded fp32 operation (no fused
 * multiply-add).  grads: DEVICE, read-only; worker w's arena starts at
 * grads + w*worker_stride (elements, multiple of 4, >= arena_elems).
 *
 * Both stages of an iteration see one gradient per worker, cut in two by the
 * GIB (Sec. 3.1), and LGP reads the stage-2 part as well.  The library reads
 * that part once where it can: with an element-granular GIB the stage-1 call
 * keeps the aggregate of the stage-2 elements in the workspace; with a
 * layer-granular GIB osp_lgp_correct does (N >= 4, replicas in sync, see
 * osp_set_keep_stage2_aggregate).  A stage-2 call that is handed the same
 * `grads` pointer and stride reuses the kept aggregate instead of reading the
 * N arenas again: between the two calls these arenas must not change.  A
 * stage-2 call with any other pointer or stride aggregates afresh.  Results
 * are the same bit for bit either way.
 */
osp_status osp_ps_aggregate_update(osp_ctx *ctx, int stage, const float *grads,
                                   int64_t worker_stride, void *stream);

/*
 * Gradient splitter (Sec. 4.5): every worker's gradient arena is separated,
 * according to the current GIB, into the important gradients G^i (stage 1) and
 * the unimportant gradients G^u (stage 2).  Each part is dense: the stage's
 * elements in arena order, nothing in between; worker w's parts start at
 * g_important + w*important_stride and g_unimportant + w*unimportant_stride
 * (DEVICE, 4-byte aligned, strides in elements, at least the part's size:
 * n_params - n_stage2 and n_stage2, see osp_n_stage2).  Either output may be
 * NULL.  These are the payloads a transport would carry in the two stages; the
 * other calls of this library read the arenas in place and do not need them.
 * Does not change the iteration state.
 */
osp_status osp_split_gradients(osp_ctx *ctx, const float *grads, int64_t worker_stride,
                               float *g_important, int64_t important_stride,
                               float *g_unimportant, int64_t unimportant_stride, void *stream);

/* osp_ps_aggregate_update(stage), stage 1 or 2, with the stage's gradients
 * arriving as the dense parts above (worker w's at packed + w*packed_stride):
 * same arithmetic in the same order, same results, same place in the order of
 * calls.  A stage 1 given this way leaves nothing for stage 2 to reuse. */
osp_status osp_ps_aggregate_update_packed(osp_ctx *ctx, int stage, const float *packed,
                                          int64_t packed_stride, void *stream);

/* The two calls above for bfloat16 gradient arenas (see the _bf16 calls below):
 * the dense parts hold bfloat16 as well, the same 16 bits moved, 2-byte
 * aligned; the packed aggregate widens them exactly and then is the fp32
 * arithmetic, so results equal those of the fp32 calls on the widened values. */
osp_status osp_split_gradients_bf16(osp_ctx *ctx, const uint16_t *grads, int64_t worker_stride,
                                    uint16_t *g_important, int64_t important_stride,
                                    uint16_t *g_unimportant, int64_t unimportant_stride,
                                    void *stream);
osp_status osp_ps_aggregate_update_packed_bf16(osp_ctx *ctx, int stage, const uint16_t *packed,
                                               int64_t packed_stride, void *stream);

/* LGP (Sec. 4.2, Eq. 6): for every stage-2 element and every worker,
 * P_{w,k} = P_{w,k} - lr g_{w,k}: the stale parameter advances by the worker's
 * own local gradient.  Stage-1 elements are not touched. */
osp_status osp_lgp_correct(osp_ctx *ctx, const float *grads, int64_t worker_stride,
                           void *stream);

/*
 * The two calls that read gradients, for gradient arenas kept in bfloat16
 * (fp32 master parameters and momentum as before): halves the N x M bytes the
 * step reads most.  Not in the paper.  grads: DEVICE, 8-byte aligned, worker
 * w's arena at grads + w*worker_stride (elements).  A bfloat16 widens to fp32
 * exactly, and everything after the load is the fp32 arithmetic above on those
 * values: the result is bit for bit that of the fp32 calls given the widened
 * gradients.  Rounding gradients to bfloat16 is the caller's business.
 * Same place in the order of calls; may be mixed with the fp32 calls from one
 * iteration to the next, not between the two stages of one iteration if the
 * kept stage-2 aggregate (element-granular GIB) is to be reused.
 */
osp_status osp_ps_aggregate_update_bf16(osp_ctx *ctx, int stage, const uint16_t *grads,
                                        int64_t worker_stride, void *stream);
osp_status osp_lgp_correct_bf16(osp_ctx *ctx, const uint16_t *grads, int64_t worker_stride,
                                void *stream);
/* The two windows (below) for bfloat16 gradient arenas. */
osp_status osp_rs_window_bf16(osp_ctx *ctx, const uint16_t *grads, int64_t worker_stride, void *stream);
osp_status osp_ics_window_bf16(osp_ctx *ctx, const uint16_t *grads, int64_t worker_stride,
                               int granularity, int64_t budget_elems, void *stream);

/* Workers receive the global parameters of a stage (Sec. 2.1.1); for stage 2
 * this is the correction of Eq. 7, which replaces the local LGP estimate by the
 * global result (taken as an overwrite, P_{w,k} = P_k).  stage: 1, 2, or 0 = both. */
osp_status osp_apply_stage(osp_ctx *ctx, int stage, void *stream);

/*
 * The two synchronization windows of an iteration (Sec. 3.1, Fig. 4) as one
 * call each.  Same arguments, same checks and, element for element, the same
 * results as the calls they stand for:
 *   osp_rs_window  = osp_ps_aggregate_update(1), osp_apply_stage(1), osp_lgp_correct
 *                    (RS: the important gradients are synchronized inside the
 *                    barrier and the workers advance their stale unimportant
 *                    parameters by LGP, Eq. 6);
 *   osp_ics_window = osp_ps_aggregate_update(2), osp_apply_stage(2), osp_split
 *                    (ICS, overlapped by the caller with the next iteration's
 *                    compute: Eq. 7, then the next GIB, Sec. 3.2).
 * When the replicas equal the PS arena as the RS window begins (after
 * osp_bind with replicas_in_sync, or after an iteration that installed both
 * stages) the windows run fused kernels: one launch per window (plus the
 * split's), no second read of data a lane already holds.  Otherwise, and
 * where the single-stage kernels are as fast (layer-granular GIB: N > 8 or
 * N x parameters > 2^25; element-granular GIB: RS window N > 16, ICS window
 * N > 8), they enqueue the single-stage kernels.  The single calls and
 * the windows may be mixed freely within the order of calls above.
 * The rule on the gradient arenas between the two stages (see
 * osp_ps_aggregate_update) applies.
 */
osp_status osp_rs_window(osp_ctx *ctx, const float *grads, int64_t worker_stride, void *stream);
osp_status osp_ics_window(osp_ctx *ctx, const float *grads, int64_t worker_stride,
                          int granularity, int64_t budget_elems, void *stream);

/* Both windows back to back on one stream: a whole iteration's synchronization
 * without overlap (what a benchmark of the arithmetic times; a training loop
 * puts the next iteration's compute between the two windows instead). */
osp_status osp_sync_step(osp_ctx *ctx, const float *grads, int64_t worker_stride, int granularity,
                         int64_t budget_elems, void *stream);

/* Inspection (each synchronizes `stream`): the fp64 layer importances I^l of
 * the last osp_split(LAYER) into imp_host[L]; the element keys (bit pattern of
 * I_k, NaN canonicalised to 0x7FC00000, padding 0xFFFFFFFF) into
 * key_host[arena_elems] (needs cfg.element_keys). */
osp_status osp_get_importance(osp_ctx *ctx, double *imp_host, void *stream);
osp_status osp_get_keys(osp_ctx *ctx, uint32_t *key_host, void *stream);

/* Plain device-to-device copy of `bytes` (multiple of 16; both pointers DEVICE,
 * 16-byte aligned, not overlapping) with the same access shape and cache policy
 * as the step's kernels.  A reference line for bandwidth measurements and the
 * known-size kernel that hardware traffic counters are calibrated against; not
 * part of the synchronization step.  At most 2^31 KiB per call. */
osp_status osp_stream_copy(void *dst, const void *src, size_t bytes, void *stream);

/* A second reference line: the traffic of osp_ps_aggregate_update's shape without
 * its arithmetic.  n_read streams (reads + s*read_stride, s < n_read) are read
 * and summed; n_rw streams (1 or 2; rw + s*rw_stride) are read and written back
 * with the sum added; n_elems elements (multiple of 4) of every stream, strides
 * in elements (multiples of 4, >= n_elems), all DEVICE and 16-byte aligned.
 * What it sustains is the ceiling of that access pattern on the machine at
 * hand.  Not part of the synchronization step. */
osp_status osp_stream_pattern(const float *reads, int32_t n_read, int64_t read_stride, float *rw,
                              int32_t n_rw, int64_t rw_stride, int64_t n_elems, void *stream);

/*
 * S(G^u) tuning (Sec. 4.1.2).  Host-only scalar functions: no context, no GPU.
 *
 * osp_ics_upper_bound: Eq. 5 as printed, U_max = b (1 + lr) T_c / N, the most
 * that fits into one iteration's compute window; bandwidth in elements per
 * second, loss_rate in [0, 1], t_compute in seconds.  Returns 0 for arguments
 * that are not finite and non-negative or for n_workers < 1.
 *
 * osp_tune_budget: Algorithm 1.  U_max is first capped at 80 % of the model;
 * epoch 1 synchronizes everything in stage 1 (returns 0 and the caller keeps
 * loss_1 as L); epoch i > 1 returns floor((1 - loss_i / L) * U_max), clamped to
 * [0, capped U_max] (a loss above L gives 0).  The result is the budget_elems
 * argument of osp_split.  Returns -1 for arguments that are not finite, a
 * non-positive L, epoch < 1 or a negative model size.
 */
double osp_ics_upper_bound(double bandwidth_elems_per_s, double loss_rate, double t_compute_s,
                           int32_t n_workers);
int64_t osp_tune_budget(int32_t epoch, double loss_i, double loss_1, double u_max,
                        int64_t model_elems);

/* Message for the last error on this context ("" if none).  With ctx == NULL,
 * the message of the last failed osp_create on this thread. */
const char *osp_last_error(const osp_ctx *ctx);

/* 1 if the last osp_lgp_correct read the stale stage-2 values once from the PS
 * arena (replicas known to be in sync) instead of once per replica; 0 otherwise.
 * For callers that account for the bytes a step really moves. */
int32_t osp_lgp_read_shared(const osp_ctx *ctx);

/* Whether osp_lgp_correct (and the RS window built from it) keeps the aggregate
 * of a layer-granular stage 2 for the stage-2 call (default: on).  On one GPU
 * with nothing overlapping the ICS this moves fewer bytes per iteration; it
 * also makes the RS window, the part inside the barrier (Sec. 3.1), a little
 * longer (its workgroups write all N replicas instead of sweeping them one by
 * one), which a caller who overlaps the ICS with compute may not want.
 * OSP_ERR_BAD_STATE between the two stages of an iteration. */
osp_status osp_set_keep_stage2_aggregate(osp_ctx *ctx, int32_t on);

/* Reuse of a kept stage-2 aggregate is decided by the `grads` pointer and stride
 * alone (see osp_ps_aggregate_update); the library cannot see whether the caller
 * has written new values into those arenas since.  A caller that has calls this
 * before the stage-2 call, which then aggregates the arenas afresh.  Host only. */
osp_status osp_drop_kept_aggregate(osp_ctx *ctx);

/* 1 if the last osp_lgp_correct kept the stage-2 aggregate; 0 otherwise.  For
 * callers that account for the bytes a step really moves. */
int32_t osp_lgp_kept_aggregate(const osp_ctx *ctx);

/* Which of the last osp_rs_window (bit 0) and osp_ics_window (bit 1) ran as a
 * fused kernel rather than as the single-stage kernels.  For reports. */
int32_t osp_windows_fused(const osp_ctx *ctx);

/* Geometry, for callers that size launches or report traffic. */
int32_t osp_chunk_elems(const osp_ctx *ctx);
int64_t osp_n_chunks(const osp_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* OSP_H */
