/*
 * ssd.h -- C ABI of the SSD-SGD parameter-update pipeline for MI355X (gfx950).
 *
 * The library runs, on one GPU, the per-iteration update path of SSD-SGD
 * ("Several Steps Delay SGD"): the parameter-server side (sum the K workers'
 * gradients, apply momentum SGD with weight decay; Eq. (server) and the
 * momentum rule of Sec. 3.2.1 of the paper) and the worker side (the GLU
 * local update of Eq. (glu-update) with grad_sync of Sec. 3.3, scheduled by
 * Algorithm 1 and Algorithm 2), over every layer tensor of a model.  The K
 * workers are K resident sets of device arrays.
 *
 * Conventions for every entry point
 *   - All data are IEEE binary32, except that the workers' gradient buffers
 *     may hold 16-bit values (ssd_config.grad_dtype, an extension: the paper's
 *     gradients are binary32).  Pointers named "device" point to GPU global
 *     memory of the configured device; all other pointers are host memory
 *     that the library reads during the call only (it keeps no reference).
 *   - Calls enqueue work on the stream given at ssd_init and return without
 *     waiting for it.  Ordering against the caller's other GPU work is stream
 *     order.  A context must be used from one host thread at a time;
 *     different contexts may be used from different threads at once.
 *   - Return value: SSD_OK (0) or a negative SSD_E* code.  Arguments are
 *     checked before anything is enqueued, so a failing call leaves the state
 *     untouched.  ssd_last_error gives a message for the last failure.
 *   - Nothing here throws or aborts across the boundary.
 */
#ifndef SSD_H
#define SSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SSD_OK 0
#define SSD_EINVAL (-1) /* null / negative / out-of-range argument            */
#define SSD_EALIGN (-2) /* a device pointer is not aligned to its element
                           size, or the workspace is not 256-byte aligned      */
#define SSD_ENOMEM (-3) /* workspace too small, or host allocation failed     */
#define SSD_EHIP (-4)   /* a HIP runtime call failed; text in ssd_last_error  */
#define SSD_ESTATE (-5) /* call not allowed in the current schedule state     */

#define SSD_MAX_WORKERS 16

/* Kinds of iteration of the worker schedule (Algorithm 1 + Algorithm 2).
 * d is the index of the steps-delay iteration (Alg. 2's loc_update). */
enum ssd_step_kind {
    SSD_STEP_WARMUP = 0,       /* SSGD iteration of the warm-up loop          */
    SSD_STEP_WARMUP_LAST = 1,  /* last warm-up iteration: w'_i = w_t taken    */
    SSD_STEP_DELAY = 2,        /* local update, no Pull                       */
    SSD_STEP_DELAY_PULL = 3    /* local update, then Pull (d % k == k-1)      */
};
/* What Algorithm 2 does with pre_weight on a local update. */
enum ssd_pre_action {
    SSD_PRE_KEEP = 0,    /* grad_sync from pre_weight, pre_weight kept        */
    SSD_PRE_INIT = 1,    /* d == 0: pre_weight initialised with w'            */
    SSD_PRE_REFRESH = 2  /* d > 0 and d % k == 0: pre_weight = w' afterwards  */
};

/* Where the weights for the next forward/backward (w_loc, Alg. 1's Broadcast
 * target) are found. */
enum ssd_w_loc_where {
    SSD_W_LOC_IS_GLOBAL = 0,  /* the global weights (warm-up stage, hand-over)  */
    SSD_W_LOC_IN_W_LOCAL = 1, /* the w_local arrays: w_loc_i is w'_i itself, or
                                 -- after a Pull iteration of ssd_step -- the
                                 local weights as broadcast before the Pull    */
    SSD_W_LOC_SEPARATE = 2    /* the w_loc arrays (after ssd_worker_pull or
                                 ssd_materialize)                              */
};

/* Element type of the workers' gradient buffers.  The paper's gradients are
 * binary32; the 16-bit types are an extension for frameworks whose backward
 * pass emits them (mixed-precision training) and cut the bytes the update
 * path reads.  A 16-bit gradient is widened to binary32 exactly (every
 * bfloat16 and binary16 value is a binary32 value) as it is loaded; the
 * arithmetic after the load is the same binary32 sequence in all three
 * cases.  rescale_grad can carry the inverse of a loss scale. */
enum ssd_grad_dtype {
    SSD_GRAD_F32 = 0,  /* IEEE binary32, 4 bytes per element                   */
    SSD_GRAD_BF16 = 1, /* bfloat16: the upper 16 bits of a binary32            */
    SSD_GRAD_F16 = 2   /* IEEE binary16                                        */
};

/* How the fused kernel marks its global loads and stores. */
enum ssd_cache_policy {
    SSD_CACHE_AUTO = 0,      /* the library's choice (see ssd_config)            */
    SSD_CACHE_STREAMING = 1, /* non-temporal: every byte of an iteration is
                                touched once and nothing fits a cache           */
    SSD_CACHE_RESIDENT = 2   /* ordinary accesses: the arrays of a small model
                                stay in the last-level cache between iterations */
};

typedef struct ssd_ctx ssd_ctx; /* opaque */

/* Configuration.  Symbols follow Table 1 of the paper. */
typedef struct {
    int32_t num_workers;   /* K, 1..SSD_MAX_WORKERS                           */
    int32_t delay_k;       /* k >= 0 delay steps; 0 = SSGD for ever           */
    int32_t warmup_iters;  /* W >= 0 SSGD iterations before the steps-delay
                              stage; Algorithm 1's wp + 1                     */
    float lr;              /* global learning rate in the servers             */
    float momentum;        /* m, momentum coefficient in the servers          */
    float wd;              /* weight decay in the servers                     */
    float lr_loc;          /* loc_lr; the paper uses 4 * lr (Sec. 4.1)        */
    float alpha;           /* weight of the local gradient, 2.0 in Sec. 4.1   */
    float beta;            /* weight of grad_sync, 0.5 in Sec. 4.1            */
    float wd_loc;          /* weight decay inside Eq. (glu-update)            */
    float rescale_grad;    /* factor on the sum of the K gradients; 1/K gives
                              the averaged gradient of Table 1                */
    int32_t num_tensors;   /* T >= 1 layer tensors                            */
    const int64_t *numel;  /* host [T], elements per tensor, each >= 1        */
    int32_t device;        /* HIP device ordinal                              */
    void *stream;          /* hipStream_t; NULL = the default stream          */
    int32_t chunk_elems;   /* elements per work chunk of the multi-tensor
                              launch; 0 = choose (256: one 64-lane wave x 4
                              floats); else a multiple of 256                 */
    int32_t waves_per_cu;  /* cap on wavefronts resident per compute unit in
                              the fused launch; 0 = the library's measured
                              choice per kernel (see ssd_lds_slice_bytes)     */
    int32_t grad_sync_exact; /* 0: grad_sync from (pre_weight - w') as printed
                              in Sec. 3.3; 1: from the exact w_minus of
                              Sec. 3.2.1, ((1 - lr*wd)*pre_weight - w')       */
    int32_t grad_dtype;    /* an ssd_grad_dtype: element type of every gradient
                              buffer passed to this context                   */
    int32_t cache_policy;  /* an ssd_cache_policy for the fused launch; 0 = the
                              library's choice: resident (ordinary accesses,
                              no cap on resident waves) if the arrays one
                              iteration touches -- K gradients, K local
                              weights, weight, momentum, pre_weight -- fit
                              the 256 MiB last-level cache of MI355X, else
                              streaming.  Results never depend on it.         */
} ssd_config;

/* Device-side state, for inspection.  All arrays are "arena" arrays of
 * arena_elems floats in which tensor t occupies
 * [tensor_offset[t], tensor_offset[t] + numel[t]).  Tensors own whole blocks
 * of chunk_elems elements, in tensor order; a tensor of at least 8192 elements
 * whose weight pointer is 16-byte aligned does not start at the beginning of
 * its first block but ((address mod 1024) / 4) elements into it, so that the
 * 256-element tiles the kernels work on are aligned 1 KiB pieces of the
 * caller's arrays as well as of these.  Worker i's w_loc array starts at
 * w_loc + i * arena_elems.  The K local-weight arrays w'_i are laid out block
 * by block: arena element a of worker i is
 *   w_local[i * w_local_worker_stride + (a / chunk_elems) * w_local_block_stride
 *           + a % chunk_elems],
 * which for up to 8 workers is the same planar form (strides arena_elems and
 * chunk_elems) and for more workers puts the K copies of a block side by side
 * (strides chunk_elems and K * chunk_elems).  The pointers stay valid
 * until ssd_destroy; the data they show are those of the work enqueued so
 * far (synchronise the stream before reading). */
typedef struct {
    int64_t iterations;     /* ssd_step calls completed (Alg. 1's num)        */
    int64_t local_updates;  /* d: local updates done by every worker          */
    int32_t in_delay_stage; /* 0 while the next ssd_step is a warm-up step    */
    int32_t has_local;      /* 1 once every worker has local weights w'_i     */
    int32_t w_local_is_global; /* 1: every w'_i equals the global weight (after
                               the end of warm-up or a Pull of ssd_step) and
                               the w_local arrays do not hold it              */
    int32_t w_loc_where;    /* where w_loc_i (what the next forward/backward
                               uses) is: an ssd_w_loc_where value             */
    int32_t chunk_elems;
    int32_t streaming;      /* 1: the fused launch uses non-temporal accesses
                               (SSD_CACHE_STREAMING), 0: ordinary ones         */
    int64_t num_chunks;
    int64_t arena_elems;
    int64_t w_local_worker_stride; /* see above                               */
    int64_t w_local_block_stride;
    const int64_t *tensor_offset; /* host [T], owned by the context           */
    float *mom;             /* device: momentum of the servers                */
    float *pre;             /* device: pre_weight (one copy: Sec. 3.3 says all
                               workers hold the same value)                   */
    float *w_local;         /* device: w'_i, K arrays (see w_local_is_global)  */
    float *w_loc;           /* device: K arrays, valid when w_loc_where says   */
} ssd_state_view;

/* Fill *cfg with the paper's settings for K workers and a global learning rate
 * lr: loc_lr = 4 * lr, alpha = 2.0, beta = 0.5 (Sec. 4.1, "Hyper-parameters");
 * rescale_grad = 1/K, the averaged gradient the servers apply (Table 1; the
 * 1/K of Eq. (server)); wd for the servers and, as Eq. (glu-update) prints the
 * same symbol, for the local update (wd_loc).  Everything else is zeroed:
 * binary32 gradients, no warm-up, delay_k = 0, the library's choices for
 * chunk_elems and waves_per_cu, stream NULL.  The caller then sets delay_k,
 * warmup_iters, momentum, the tensor list, device and stream.  Host-only. */
int ssd_config_defaults(ssd_config *cfg, int32_t num_workers, float lr, float wd);

/* Bytes of device workspace ssd_init needs for this configuration (state
 * arrays, chunk table, pointer tables).  Host-only; touches no GPU. */
int ssd_workspace_bytes(const ssd_config *cfg, size_t *bytes);

/* Create a context (Algorithm 1, initialisation: global weight w_0 given,
 * num = 0; momentum starts at 0).
 *   weights   host [T] of device pointers: the global weights w_t, owned by
 *             the caller, updated in place by every server update; must stay
 *             valid until ssd_destroy.  Any 4-byte alignment works; 16 bytes
 *             (for the weight and every gradient pointer of a tensor) select
 *             the 128-bit path.  Tensors need not start at 1 KiB boundaries
 *             for full speed: the state arrays are laid out to follow the
 *             weight pointers' 1 KiB grid (see ssd_state_view), which pays
 *             off when the gradient buffers share that phase, as buffers laid
 *             out like the weights do.
 *   workspace device memory of at least ssd_workspace_bytes, 256-byte
 *             aligned, owned by the caller, used exclusively by the context
 *             until ssd_destroy.
 * Enqueues the clearing of the momentum and of the other state arrays (if
 * warmup_iters == 0 and delay_k > 0, w'_i = w_0 is recorded, not copied: see
 * ssd_state_view.w_local_is_global).  On failure *out is NULL and
 * ssd_last_error(NULL) has the reason. */
int ssd_init(const ssd_config *cfg, float *const *weights, void *workspace,
             size_t workspace_bytes, ssd_ctx **out);

/* Server side of one iteration (Eq. (server); momentum rule of Sec. 3.2.1):
 *   S = g_0 + g_1 + ... + g_{K-1} (in this order), g = rescale_grad * S,
 *   mom = m*mom - lr*(g + wd*w),  w = w + mom.
 *   grads  host [K] of host [T] of device pointers, read-only gradients of
 *          worker i, tensor t, numel[t] elements of ssd_config.grad_dtype
 *          each, aligned to the element size.  Placement advice, measured on
 *          MI355X: K buffers that lie an exact multiple of 256 MiB apart cost
 *          4 % (steps-delay kernels) to 9 % (warm-up kernel) at K = 8; any
 *          other distance, e.g. one 64 MiB unit more, does not.
 * Does not advance the schedule.  (Materialises first, see ssd_materialize.) */
int ssd_server_aggregate_update(ssd_ctx *ctx, const void *const *const *grads);

/* One call of Algorithm 2 (GLU) for one worker, on its local weight w'_i:
 *   grad_sync = (pre_weight - w') * (1-m)/(lr*k)            (Sec. 3.3; see
 *                                         ssd_config.grad_sync_exact)
 *   pre_weight initialised with w' on the worker's first call, refreshed
 *   with w' (value before this update) when loc_update > 0 and
 *   loc_update % k == 0,
 *   w' = w' - lr_loc*(alpha*g_i + wd_loc*w' + beta*grad_sync)  (Eq. glu-update)
 *   grads_i  host [T] of device pointers, worker i's gradients.
 * Needs delay_k > 0 and a worker that has pulled (SSD_ESTATE otherwise).
 * Workers must advance in lock step: a worker may be at most one local update
 * ahead of the slowest one (SSD_ESTATE otherwise); pre_weight is shared. */
int ssd_worker_glu_update(ssd_ctx *ctx, int32_t worker, const void *const *grads_i);

/* Pull of Algorithm 1 for one worker: w_loc_i = w'_i (the weights the next
 * forward/backward uses), then w'_i = w_t (current global weight).  For a
 * worker without local weights yet (the hand-over at the end of the warm-up
 * stage) both become w_t. */
int ssd_worker_pull(ssd_ctx *ctx, int32_t worker);

/* One full iteration of Algorithm 1 for the server and all K workers, as one
 * fused launch: warm-up iterations run the server update only; steps-delay
 * iterations run the server update and the K GLU updates.  The hand-over at
 * the end of warm-up (w'_i = w_t) and the Pull when d % k == k-1 (w_loc_i =
 * w'_i, then w'_i = w_t) move no data: the context records that every w'_i is
 * the global weight (ssd_state_view.w_local_is_global) and the next iteration
 * takes it from there.  In values, equivalent bit for bit to
 * ssd_server_aggregate_update + K x ssd_worker_glu_update (+ K x
 * ssd_worker_pull).  Needs all workers at the same local update count.
 *
 * Graph capture.  Once a set of gradient pointers has been used on a stream
 * (the context keeps the pointer tables of the last 8 distinct sets on the
 * device), a further ssd_step with it on that stream enqueues exactly one
 * kernel launch: no copy, no memset, no allocation, no wait.  Such calls may be
 * recorded into a HIP graph by capturing the stream.  A graph that holds whole
 * k-cycles starting at a cycle boundary (local_updates % k == 0, after at
 * least one earlier cycle) can be replayed any number of times: the recorded
 * flags return to their values at the start of the cycle, so each replay is
 * the next k iterations.  Replays do not advance the counters that
 * ssd_get_state reports, and the captured gradient sets must not be evicted
 * (use at most 8 distinct sets while the graph lives).  The hyper-parameters
 * travel as kernel arguments, so a captured launch keeps the learning rates of
 * the time of capture: capture again after ssd_set_lr. */
int ssd_step(ssd_ctx *ctx, const void *const *const *grads);

/* Write out the state that ssd_step only records: if w_local_is_global, copy
 * the broadcast local weights into the w_loc arrays and the global weight into
 * every w'_i (afterwards w_local_is_global = 0, w_loc_where = SEPARATE).  The
 * piecewise calls do this themselves when needed; no-op otherwise. */
int ssd_materialize(ssd_ctx *ctx);

/* Change the learning rates (schedules).  lr is the global learning rate in
 * the parameter servers (Table 1) and therefore also the one inside grad_sync,
 * which inverts the servers' momentum recursion (Sec. 3.2.1, Sec. 3.3:
 * grad_sync = (pre_weight - w') * (1-m)/(lr*k)); lr_loc is loc_lr of
 * Eq. (glu-update).  The paper changes neither during a run; here both take
 * effect from the next call on, and the constant (1-m)/(lr*k) is formed
 * again from the new lr.  lr = 0 with delay_k > 0 is SSD_EINVAL.  Enqueues
 * nothing unless per-tensor multipliers are set (then one small upload), so a
 * schedule may call it every iteration. */
int ssd_set_lr(ssd_ctx *ctx, float lr, float lr_loc);

/* Per-tensor multipliers, as optimisers of deep-learning frameworks keep them
 * (e.g. no weight decay on biases and normalisation parameters; the paper is
 * silent on them): tensor t uses lr*lr_mult[t] and lr_loc*lr_mult[t] as its
 * learning rates (also inside grad_sync) and wd*wd_mult[t], wd_loc*wd_mult[t]
 * as its weight decays, each product one binary32 multiplication.  Host arrays
 * [T], values >= 0; NULL = all ones.  A tensor with lr_mult 0 is frozen and
 * its grad_sync is 0.  Takes effect for the calls that follow. */
int ssd_set_tensor_multipliers(ssd_ctx *ctx, const float *lr_mult, const float *wd_mult);

/* Enqueue the following calls on another stream (NULL = the default stream).
 * The library adds no synchronisation between streams except for its own
 * pointer tables: work on different streams that touches the same arrays --
 * e.g. the server update of the next iteration against a Pull still reading
 * the global weight -- must be ordered by the caller with events.  This is
 * what lets the server update and the local updates of one iteration run
 * side by side, as in the execution order of the paper's Fig. 3(b) (Push and
 * local update only read the gradient).  Every stream ever given to a context
 * must stay alive until ssd_destroy: the context may have to wait for it when
 * it reuses a pointer table that a launch on that stream has read. */
int ssd_set_stream(ssd_ctx *ctx, void *stream);

/* Fill *out (host).  Does not synchronise. */
int ssd_get_state(ssd_ctx *ctx, ssd_state_view *out);

/* Message of the last failing call on this context; ctx == NULL: of the last
 * failing ssd_init / ssd_workspace_bytes on this thread.  Never NULL. */
const char *ssd_last_error(const ssd_ctx *ctx);

/* Release host resources.  Work already enqueued must have finished or the
 * caller must synchronise the stream first; workspace and weights are the
 * caller's to free afterwards.  NULL is allowed. */
void ssd_destroy(ssd_ctx *ctx);

/* ---- for callers that cannot allocate ----------------------------------- */

/* The server side of one iteration -- the same rule, rounding sequence and
 * multi-tensor launch as ssd_server_aggregate_update -- for callers that
 * cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  There is no context and no workspace: the
 * call allocates nothing on the host or the device, calls no hipMalloc /
 * hipFree and no allocating library routine.  The tables its launch needs sit
 * in a static device array inside the library, 2,260,992 bytes per GPU
 * (163,840 of tensor records + 2,097,152 of block table), held by every GPU
 * the library runs on until the process ends.  Hence the limits: at most
 * SSD_NOALLOC_MAX_TENSORS tensors and SSD_NOALLOC_MAX_BLOCKS blocks of 256
 * elements (a tensor of n elements takes ceil(n / 256) blocks; 268,435,456
 * elements if all are multiples of 256); a larger model is SSD_EINVAL.
 *   numel     host [T], elements per tensor, each >= 1
 *   weights   host [T] of device pointers, w_t, updated in place
 *   momentum  host [T] of device pointers, the servers' momentum, updated in
 *             place; the caller owns it (zero it before the first iteration)
 *   grads     host [K][T] of device pointers, binary32 gradients, read-only
 *   lr, m, wd, rescale_grad  as in ssd_config
 * All device pointers 4-byte aligned (SSD_EALIGN); tensors whose pointers are
 * all 16-byte aligned take 128-bit accesses.  Enqueues a few small launches
 * that write the tables and one update launch on `stream` and returns without
 * waiting.  Every call on a GPU uses that GPU's one static array and
 * overwrites what the call before left there (nothing in it needs clearing:
 * a call writes every entry it reads): calls on one stream follow each other
 * correctly, calls that overlap on one GPU -- other streams, other host
 * threads -- race.  Errors as everywhere: checked before anything is
 * enqueued; message from ssd_last_error(NULL). */
#define SSD_NOALLOC_MAX_TENSORS 1024
#define SSD_NOALLOC_MAX_BLOCKS 1048576
int ssd_server_aggregate_update_noalloc(int32_t num_workers, int32_t num_tensors, const int64_t *numel,
                                        float *const *weights, float *const *momentum,
                                        const float *const *const *grads, float lr, float m, float wd,
                                        float rescale_grad, int32_t device, void *stream);

/* ---- host-only helpers (no GPU), used by the calls above ---------------- */

/* Kind of iteration number `iteration` (0-based) and pre_weight action, for
 * W warm-up iterations, delay k, and d local updates done so far.
 * Returns an ssd_step_kind, or SSD_EINVAL. */
int ssd_step_kind_of(int64_t iteration, int32_t warmup_iters, int32_t delay_k,
                     int64_t local_updates, int32_t *pre_action);

/* Bytes of LDS that each single-wave workgroup of the fused launch is given,
 * and never touches, so that at most waves_per_cu of them fit a compute unit
 * with lds_bytes_per_cu bytes of LDS (163840 on MI355X; ssd_init reads the
 * device's own value).  LDS is handed out in 128 granules per compute unit, so
 * the slice is floor(128 / waves_per_cu) granules; the compute unit then holds
 * floor(128 / floor(128 / waves_per_cu)) waves, which is waves_per_cu itself
 * for 1..12, 14 and 16 (13 gives 14, 15 gives 16).  0 for waves_per_cu = 0 or
 * >= 32 (no cap); SSD_EINVAL for a negative count or an LDS size that is not a
 * positive multiple of 128. */
int ssd_lds_slice_bytes(int32_t waves_per_cu, int32_t lds_bytes_per_cu);

/* Work chunk of the multi-tensor launch: `len` elements of tensor `tensor`
 * starting at element `offset` of that tensor. */
typedef struct {
    int32_t tensor;
    int32_t len;
    int64_t offset;
} ssd_chunk;

/* Split T tensors into chunks of at most chunk_elems elements (chunk_elems a
 * positive multiple of 256; 0 = the library's choice).  Every
 * element of every tensor lies in exactly one chunk; chunks of a tensor start
 * at multiples of chunk_elems.  Writes up to `capacity` chunks to `out` (may
 * be NULL to count only) and the total number to *count; *chunk_elems_used
 * (may be NULL) receives the chunk size. */
int ssd_plan_chunks(const int64_t *numel, int32_t num_tensors, int32_t chunk_elems,
                    ssd_chunk *out, int64_t capacity, int64_t *count,
                    int32_t *chunk_elems_used);

/* The arena layout and the blocks of the launch that ssd_init would choose for
 * this configuration and these weight pointers.  Host arithmetic on the
 * pointer VALUES only: nothing is dereferenced and no GPU is touched.  It
 * differs from ssd_plan_chunks by the lead-in of large tensors (see
 * ssd_state_view): a block is chunk_elems consecutive arena elements, and the
 * part of it that belongs to the tensor may start after the block's start.
 *   tensor_offset  [T] or NULL: arena element of each tensor's element 0, as
 *                  ssd_get_state reports it
 *   out, capacity  NULL, or room for `capacity` blocks: block b covers `len`
 *                  elements of tensor `tensor` from element `offset` on
 *   num_blocks     NULL, or the number of blocks (workgroups of a launch)
 *   bytes          NULL, or the workspace this layout needs; never more than
 *                  ssd_workspace_bytes, which holds for every alignment
 * Every element of every tensor lies in exactly one block. */
int ssd_plan_arena(const ssd_config *cfg, float *const *weights, int64_t *tensor_offset,
                   ssd_chunk *out, int64_t capacity, int64_t *num_blocks, size_t *bytes);

/* ---- measurement aid ---------------------------------------------------- */

/* Plain copy of n floats, device src -> device dst, on `stream`, with the same
 * 128-bit streaming loads and stores the update kernels use: 4*n bytes read,
 * 4*n bytes written, nothing else.  It is the known-size kernel against which
 * hardware memory counters are scaled, and a practical bandwidth ceiling.
 * n >= 0 and a multiple of 4; both pointers 16-byte aligned (SSD_EALIGN). */
int ssd_probe_copy(const float *src, float *dst, int64_t n, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SSD_H */
