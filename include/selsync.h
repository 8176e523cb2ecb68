/*
 * selsync.h -- C ABI of the MI355X-native SelSync per-step hot path.
 *
 * SelSync ("Accelerating Distributed ML Training via Selective Synchronization")
 * decides every training step between a purely local SGD update and a
 * synchronisation of all workers, by tracking how much the squared gradient norm
 * has changed (Sec. III-A/B, Alg. 1).  This library runs that per-step path for K
 * worker replicas resident in the HBM of ONE gpu (gfx950):
 *
 *   a1  ||g_k||^2 for every worker k, one fused multi-tensor reduction   (Alg. 1 line 8)
 *   a2  windowed-EWMA smoothing, Delta(g_i) of Eq. 2, flag_k = Delta_k >= delta,
 *       sync = OR_k flag_k                                               (Sec. III-A/B, Alg. 1 lines 8, 10-13)
 *   a3  fused SGD(momentum, weight decay) local update                   (Alg. 1 line 9, Sec. IV-A recipes)
 *   a4  parameter aggregation: mean over the K replicas written to the
 *       global model and back into every replica                         (Alg. 1 lines 14-15)
 *
 * Conventions
 *   - Every function returns an int32_t status (SELSYNC_OK == 0).  No exception
 *     crosses the boundary.  selsync_last_error() gives a message for the last
 *     failure on that context.
 *   - "device pointer" = HIP device memory on the GPU that was current when the
 *     context was created.  "host pointer" = ordinary host memory.
 *   - The CALLER owns every tensor buffer; the library never frees or reallocates
 *     them.  Descriptors are copied at plan time; the data pointers must stay valid
 *     (and the memory allocated) until all work enqueued with that plan has finished.
 *   - Tensors are contiguous.  Pointers need only element alignment.  When all buffers of
 *     a tensor (its gradient, parameter, momentum, ...) sit at the same position relative
 *     to 16-byte alignment -- always true for 16-byte aligned buffers, and for views at the
 *     same element offset into aligned arenas -- the library peels up to 3 elements and
 *     runs 128-bit accesses over the rest; otherwise that tensor is processed element by
 *     element (same results, lower bandwidth).  Work is cut into pieces where a tensor's
 *     ADDRESSES cross multiples of the piece size (1 KiB of fp32 by default), so a tensor
 *     may start anywhere in an arena; it is fastest when the buffers of a tensor also
 *     share their position relative to that size, as separately allocated tensors do.
 *   - Buffers that are written (params, momenta, masters, global) must not overlap
 *     each other or the gradients; this is checked at plan time.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All work
 *     is ordered on that stream.  Per-step calls never allocate memory and never
 *     synchronise the host unless `blocking` is non-zero; non-blocking per-step calls
 *     enqueue kernels only (no copies, no memsets), so a caller may capture them in a
 *     HIP graph and replay it (timing events must be off while capturing).
 *   - One context may be used by one host thread at a time.
 */
#ifndef SELSYNC_H
#define SELSYNC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ---------------------------------------------------------- */
#define SELSYNC_OK                  0
#define SELSYNC_ERR_INVALID_ARG     1   /* null pointer, bad count, bad config value, overlapping buffers */
#define SELSYNC_ERR_SHAPE_MISMATCH  2   /* lists differ in tensor count or numel */
#define SELSYNC_ERR_DTYPE           3   /* unsupported dtype or dtype combination */
#define SELSYNC_ERR_OOM             4   /* host or device allocation failed */
#define SELSYNC_ERR_HIP             5   /* a HIP runtime call failed (see selsync_last_error) */
#define SELSYNC_ERR_NOT_DEVICE_MEM  6   /* a tensor pointer is not device memory of the context's GPU */
#define SELSYNC_ERR_STATE           7   /* call not valid for this plan/context (e.g. no gradients bound) */
#define SELSYNC_ERR_TOO_LARGE       8   /* input beyond the fixed capacity of an allocation-free entry point */
#define SELSYNC_WARN_NONFINITE    100   /* blocking read saw a non-finite ||g||^2; results are still written */

/* ---- element types --------------------------------------------------------- */
#define SELSYNC_F32   0   /* IEEE binary32 */
#define SELSYNC_BF16  1   /* bfloat16: upper 16 bits of binary32 */

/* ---- plain-data descriptors -------------------------------------------------- */

/* One contiguous tensor.  data: device pointer (may be NULL only if numel == 0). */
typedef struct selsync_tensor {
    void   *data;
    int64_t numel;
    int32_t dtype;      /* SELSYNC_F32 or SELSYNC_BF16 */
    int32_t reserved;   /* must be 0 */
} selsync_tensor;

/* A list of tensors (one model replica's gradients, parameters, ...).  `tensors`
 * is a HOST pointer to `count` descriptors; it is read during the call only. */
typedef struct selsync_tensor_list {
    const selsync_tensor *tensors;
    int32_t count;
    int32_t reserved;   /* must be 0 */
} selsync_tensor_list;

/* Inputs of Alg. 1 that concern the tracker, plus the smoothing constants of Sec. III-A. */
typedef struct selsync_config {
    int32_t num_workers;   /* K >= 1: replicas held on this GPU (the cluster size N of Alg. 1)        */
    int32_t window;        /* EWMA window in iterations, >= 1 (the paper uses 25); 0 selects 25        */
    double  delta;         /* threshold on the relative gradient change, >= 0 (+inf allowed)          */
    double  alpha;         /* smoothing factor in (0,1]; <= 0 selects num_workers/100 (Sec. III-A)     */
} selsync_config;

/* Hyper-parameters of the local update (Alg. 1 line 9 with the Sec. IV-A recipes):
 *   gh = grad_scale*g;  d = gh + weight_decay*w;  m = first ? d : momentum*m + d;  w = w - lr*m
 * evaluated in fp32 with one rounding per operation (no fused multiply-add).
 * With nesterov = 1 the step direction is d + momentum*m (m the NEW buffer) instead of m.
 * On a plan created without momentum buffers the update is w = w - lr*d (plain SGD, the
 * Transformer recipe): momentum must be 0 and nesterov 0 there. */
typedef struct selsync_sgd {
    float   lr;
    float   momentum;
    float   weight_decay;
    float   grad_scale;    /* multiplies every gradient element before use (also in the norm); 1 = none */
    int32_t first_step;    /* 1: momentum buffers are uninitialised (m = d); 0: they are valid;
                              -1: decide automatically (first local update since create/reset).  The
                              automatic choice is made on the host when the call ENQUEUES its work,
                              from a per-context count of enqueued updates: a launch recorded into a
                              HIP graph keeps the value it was recorded with on every replay, so
                              pass 0 or 1 explicitly in code that is captured                          */
    int32_t nesterov;      /* 0 or 1; 1 needs momentum > 0                                             */
} selsync_sgd;

/* Hyper-parameters of the Adam variant of the local update (the AlexNet recipe of Sec. IV-A
 * uses Adam with a fixed learning rate):
 *   gh = grad_scale*g; gd = gh + weight_decay*w; m = b1*m + (1-b1)*gd; v = b2*v + ((1-b2)*gd)*gd;
 *   w = w - (lr*(m/bc1)) / (sqrt(v/bc2) + eps),   bc1 = 1 - b1^t, bc2 = 1 - b2^t
 * in fp32 with one rounding per operation and correctly rounded division / square root.
 * The betas are doubles: 1-b and 1-b^t are formed in double and rounded once to fp32. */
typedef struct selsync_adam {
    double  beta1, beta2;  /* in [0, 1)                                                            */
    float   lr;
    float   eps;
    float   weight_decay;  /* added to the gradient (L2 form)                                       */
    float   grad_scale;
    int64_t step;          /* 1-based step t of the bias corrections; <= 0: local updates since
                              create/reset, plus one.  At t = 1 the moment buffers are taken as zero */
} selsync_adam;

/* Cumulative counters (LSSR is Eq. 4; max_delta is the extremum M of Sec. III-B over finite values). */
typedef struct selsync_stats {
    int64_t steps_local;
    int64_t steps_sync;
    double  lssr;          /* steps_local / (steps_local + steps_sync); NaN before the first step */
    double  max_delta;
    int64_t nonfinite_steps;   /* steps on which some worker's ||g||^2 was not finite */
} selsync_stats;

/* Table-geometry knobs (all kernels are bandwidth bound; these exist for measurement and to let
 * tests reach the multi-tile loops with small inputs).  A value <= 0 keeps the built-in default,
 * except nontemporal, whose default is a negative value. */
typedef struct selsync_tuning {
    int32_t chunk_elems;       /* elements per piece of the update/norm chunk table (multiple of 256;
                                  default 256: one 128-bit access per lane and stream)                  */
    int32_t nontemporal;       /* 1: streaming (non-temporal) loads/stores; 0: plain; <0 default:
                                  streaming when the replicas' working set is 128 MiB or more           */
    int32_t agg_chunk_elems;   /* elements per piece of the aggregation table used by launches that follow
                                  the device-side decision (multiple of 256; default 4096).  Pieces under
                                  1024 elements run on one-wavefront workgroups, larger ones on 256 threads */
    int32_t ga_chunk_elems;    /* likewise for the gradient-aggregation update (default 4096)             */
} selsync_tuning;

typedef struct selsync_ctx  selsync_ctx;    /* opaque: tracker state, counters, workspace owner */
typedef struct selsync_plan selsync_plan;   /* opaque: chunk tables for one binding of tensor lists */

/* ---- lifecycle --------------------------------------------------------------- */

/* Create a context on the current HIP device: allocates the device-side tracker
 * state (K windows, counters) and a pinned host mirror.  *out is set on success. */
int32_t selsync_create(const selsync_config *cfg, selsync_ctx **out);

/* Waits for the device, frees everything the context owns.  Plans made from it must be
 * destroyed first.  NULL is accepted. */
int32_t selsync_destroy(selsync_ctx *ctx);

/* Clear windows, previous smoothed values, counters and the automatic first-step
 * marker, ordered on `stream`. */
int32_t selsync_reset(selsync_ctx *ctx, void *stream);

/* Change delta (the slider of Sec. III-B) for subsequent steps, ordered on `stream`. */
int32_t selsync_set_delta(selsync_ctx *ctx, double delta, void *stream);

/* Set launch-shape knobs used by plans created afterwards. */
int32_t selsync_set_tuning(selsync_ctx *ctx, const selsync_tuning *t);

/* Message for the last error on this context (never NULL; valid until the next call). */
const char *selsync_last_error(const selsync_ctx *ctx);

/* Static name of a status code. */
const char *selsync_status_string(int32_t status);

/* ---- plan -------------------------------------------------------------------- */

/*
 * Bind tensor lists and build the chunk tables (host) and upload them (device);
 * allocates the per-chunk partial-sum workspace.  All arrays of lists are HOST
 * pointers to K = num_workers lists.
 *
 *   grads   [K] gradients g_k.           F32, or BF16 in mixed mode.  May be NULL: then only
 *                                         selsync_aggregate_params is valid on the plan.
 *   params  [K] worker replicas w_k.     F32; in mixed mode the BF16 working copies.
 *   momenta [K] momentum buffers m_k.    F32.  NULL when grads is NULL.  NULL with grads given makes a
 *                                         momentum-free plan: 12 instead of 20 bytes move per
 *                                         parameter; SGD entry points (gradient aggregation included)
 *                                         then require momentum = 0, and the Adam entry points return STATE.
 *   master  [K] fp32 master parameters.  NULL in fp32 mode; required in mixed mode.
 *   global      the global model.        F32 (the fp32 master in mixed mode).
 *   global_lowp BF16 copy of the global model; NULL in fp32 mode, required in mixed mode.
 *
 * Every list must have the same tensor count and per-tensor numel.  Mixed mode is
 * selected by master != NULL.  Errors: INVALID_ARG, SHAPE_MISMATCH, DTYPE,
 * NOT_DEVICE_MEM, OOM, HIP.  On error *out is NULL and nothing is leaked.
 */
int32_t selsync_plan_create(selsync_ctx *ctx,
                            const selsync_tensor_list *grads,
                            const selsync_tensor_list *params,
                            const selsync_tensor_list *momenta,
                            const selsync_tensor_list *master,
                            const selsync_tensor_list *global,
                            const selsync_tensor_list *global_lowp,
                            selsync_plan **out);

/* Waits for the device and frees the plan.  NULL is accepted. */
int32_t selsync_plan_destroy(selsync_plan *plan);

/* Sizes of a plan: tensors per replica, parameters per replica, chunks of the
 * update table (all replicas) and of the aggregation table.  Any output may be NULL. */
int32_t selsync_plan_info(const selsync_plan *plan, int32_t *num_tensors, int64_t *num_params,
                          int32_t *update_chunks, int32_t *aggregate_chunks);

/*
 * Pure host helper (no GPU needed): the chunking rule of the multi-tensor chunk table
 * for ONE replica.  Tensors are cut where their ADDRESSES cross multiples of the chunk size
 * (chunk_elems elements; <= 0: the default): lead_elems[t] in [0, chunk_elems) says how many
 * elements past such an address tensor t starts (NULL: all 0, i.e. cutting from element 0),
 * so the first piece has up to chunk_elems - lead elements, then full pieces, then one
 * shorter last piece; empty tensors produce no chunk.  (A plan takes the lead from the
 * device addresses of the bound tensors.)  Writes up to `capacity` entries of
 * (tensor index, first element, element count) to the HOST arrays (each may be NULL) and
 * the total number of chunks to *num_chunks.
 */
int32_t selsync_chunk_table_preview(const int64_t *numel, const int32_t *lead_elems, int32_t num_tensors,
                                    int32_t chunk_elems, int32_t capacity, int32_t *tensor_out,
                                    int64_t *offset_out, int32_t *count_out, int32_t *num_chunks);

/* ---- the per-step path ---------------------------------------------------------- */

/*
 * RelativeGradChange for all K workers (Alg. 1 lines 8, 10-13; Eq. 2; Sec. III-A/B):
 * x_k = ||grad_scale*g_k||^2 over every tensor of worker k (fp64 accumulation in a fixed
 * order: the same bits on every run for tensors at the same addresses modulo the chunk
 * size; another placement regroups the sum, a difference of about 1e-16 relative),
 * pushed into worker k's window; S_k = weight-normalised EWMA over the
 * window; Delta_k = |S_k - S_k_prev| / S_k_prev; flag_k = Delta_k >= delta;
 * sync = OR_k flag_k; the local/sync counters advance.  The decision stays on the
 * device for selsync_aggregate_params.  If `blocking` != 0 the call waits for the
 * stream and fills the HOST outputs (each may be NULL): norm_sq_out[K], delta_out[K],
 * flags_out[K], sync_out[1]; it then returns SELSYNC_WARN_NONFINITE if some x_k was
 * not finite (that worker's Delta is +inf and its flag is set).
 */
int32_t selsync_track_grad_change(selsync_ctx *ctx, selsync_plan *plan, float grad_scale, void *stream,
                                  int32_t blocking, double *norm_sq_out, double *delta_out,
                                  int32_t *flags_out, int32_t *sync_out);

/*
 * Local update of all K replicas in place (Alg. 1 line 9; unconditional).  Mixed mode
 * updates the fp32 masters and rewrites the BF16 copies by round-to-nearest-even.
 * lr == 0 leaves every parameter bit-unchanged.
 */
int32_t selsync_local_step(selsync_ctx *ctx, selsync_plan *plan, const selsync_sgd *sgd, void *stream);

/*
 * Parameter aggregation (Alg. 1 lines 14-15): wbar = (sum_k w_k)/K in fp64, rounded
 * once to fp32, written to the global model and to all K replicas (mixed mode: masters
 * averaged, every BF16 copy refreshed).  Momentum buffers are not touched.
 *   mode 0: only if the device-side decision of the last tracking call is "sync"
 *           (the kernel is launched and exits at once otherwise);
 *   mode 1: always.
 * Under mode 0 the kernel reads the decision word on the device every time it runs, also when
 * replayed from a HIP graph after selsync_set_delta: nothing the host knows about the threshold
 * is ever baked into whether the launch aggregates.  Only the launch SHAPE follows the host's
 * expectation: a launch that will usually exit (mode 0 under a positive threshold) is built to
 * exit cheaply; one expected to work (mode 1, or the last decision was enqueued under a threshold
 * of 0, where every step synchronises) is built for bandwidth.
 */
int32_t selsync_aggregate_params(selsync_ctx *ctx, selsync_plan *plan, int32_t mode, void *stream);

/*
 * One whole iteration of Alg. 1 for all K workers: tracking and local update fused
 * into ONE pass over the gradients (g is read once), then the predicated aggregation.
 * Results are identical to selsync_track_grad_change + selsync_local_step +
 * selsync_aggregate_params(mode 0) in that order.  Outputs as for tracking.
 * When the context's threshold is 0 (every step synchronises) and `stream` is not being captured
 * into a HIP graph, the call runs selsync_step_bsp's single pass instead: same results, fewer bytes.
 */
int32_t selsync_step(selsync_ctx *ctx, selsync_plan *plan, const selsync_sgd *sgd, void *stream,
                     int32_t blocking, double *norm_sq_out, double *delta_out,
                     int32_t *flags_out, int32_t *sync_out);

/*
 * One fully synchronous iteration in a single pass over the data (Sec. III-B: a threshold of 0
 * turns SelSync into BSP, every step synchronises): every worker's ||grad_scale*g_k||^2, every
 * worker's local update (Alg. 1 line 9) and the mean of the UPDATED parameters written to the
 * global model and to all K replicas (Alg. 1 lines 14-15) -- 20*K + 4 bytes per parameter instead of
 * the 28*K + 4 of selsync_step's update pass plus aggregation pass.  The aggregation is
 * UNCONDITIONAL: it does not wait for, or depend on, the tracker's decision.  The tracker still runs
 * afterwards on this pass's norms (window, Delta, flags, counters under the context's threshold), so
 * with a threshold of 0 the call is selsync_step exactly: the same bits in every tensor, and the same
 * bits in the norms when the buffers of each tensor share their address modulo 1 KiB (another
 * placement regroups the fp64 sum, about 1e-16 relative).  selsync_step itself takes this path when
 * the context's threshold is 0 and `stream` is not being captured.  SGD forms only (momentum,
 * Nesterov, momentum-free plans); outputs as for selsync_track_grad_change.
 */
int32_t selsync_step_bsp(selsync_ctx *ctx, selsync_plan *plan, const selsync_sgd *sgd, void *stream,
                         int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                         int32_t *sync_out);

/* ---- variant: Adam local update (Sec. IV-A, AlexNet recipe) ---------------------------------- */

/*
 * Bind second-moment buffers v[K] (fp32, same shapes as the momenta, which then serve as the
 * first moment) to a plan that has gradients.  Caller-owned device memory; must not overlap
 * any other buffer of the plan; a tensor whose momentum buffer is 16-byte aligned must have a
 * 16-byte aligned second-moment buffer.  Waits for the device.
 */
int32_t selsync_plan_bind_second_moment(selsync_plan *plan, const selsync_tensor_list *second_moment);

/* Adam update of all K replicas in place (the local update of Alg. 1 line 9 with Adam). */
int32_t selsync_local_step_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *adam, void *stream);

/* One whole iteration with Adam as the local update: fused update + tracking pass over the
 * gradients, tracker, predicated parameter aggregation (moment buffers are not averaged).
 * Outputs as for selsync_track_grad_change. */
int32_t selsync_step_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *adam, void *stream,
                          int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                          int32_t *sync_out);

/* selsync_step_bsp with Adam as the update: one pass, unconditional aggregation of the updated
 * parameters, moment buffers stay per worker (28*K + 4 instead of 36*K + 4 bytes per parameter).
 * selsync_step_adam takes this path when the context's threshold is 0 and `stream` is not being
 * captured. */
int32_t selsync_step_bsp_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *adam, void *stream,
                              int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                              int32_t *sync_out);

/* ---- variant: gradient aggregation (Sec. III-C) ------------------------------------------ */

/*
 * Update of all K replicas under gradient aggregation.  When the decision is "sync"
 * (mode 0: the device-side decision of the last tracking call; mode 1: always), the scaled
 * gradients are averaged over the workers, gbar = fl32((sum_k (double)fl32(grad_scale*g_k))/K),
 * and EVERY worker applies gbar to its OWN parameters and momentum; otherwise every worker
 * applies its own gradient (the plain local update).  Replicas that have drifted apart stay
 * apart -- the behaviour the paper contrasts with parameter aggregation.  The global model is
 * not written.  Counts as a local update for the automatic first-step marker.
 */
int32_t selsync_ga_update(selsync_ctx *ctx, selsync_plan *plan, const selsync_sgd *sgd, int32_t mode,
                          void *stream);

/* One iteration with gradient aggregation: tracking pass over the gradients (a1 + a2), then
 * selsync_ga_update(mode 0).  Outputs as for selsync_track_grad_change. */
int32_t selsync_step_ga(selsync_ctx *ctx, selsync_plan *plan, const selsync_sgd *sgd, void *stream,
                        int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                        int32_t *sync_out);

/*
 * Gradient aggregation with Adam as the update (Sec. III-C with the Adam recipe of Sec. IV-A): on "sync"
 * every worker feeds the mean gradient to its OWN Adam state (first and second moments stay per worker and
 * are not averaged), otherwise its own gradient.  Needs bound second-moment buffers.  mode as above.
 */
int32_t selsync_ga_update_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *adam, int32_t mode,
                               void *stream);

/* One iteration: tracking pass over the gradients, then selsync_ga_update_adam(mode 0). */
int32_t selsync_step_ga_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *adam, void *stream,
                             int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                             int32_t *sync_out);

/* ---- for callers that cannot allocate ------------------------------------------------------ */

/*
 * For callers that cannot call hipMalloc -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation: the squared gradient norms of selsync_track_grad_change,
 *     x_k = || fl32(grad_scale * g_k) ||^2   over every tensor of worker k, fp64 accumulation,
 * with NO context, NO plan and NO allocation of any kind (no hipMalloc/hipFree, no memset, no
 * copy: kernel launches on `stream` only).  The per-piece partial sums live in a fixed 8 MiB
 * array in the library's device image, one copy per GPU, kept until the process ends.
 *
 *   grads        HOST array of num_workers lists (HOST descriptors, read during the call only) of
 *                DEVICE tensors on the current GPU; every list the same count and per-tensor numel,
 *                all tensors F32 or all BF16; element alignment suffices (16-byte aligned fp32 /
 *                8-byte aligned bf16 tensors take 128-/64-bit loads).  Each tensor must lie inside
 *                one device allocation (checked).
 *   norm_sq_out  DEVICE array of num_workers doubles, written by the last kernel on `stream`.
 *
 * Limits: num_workers <= 64 and, over all workers, sum of ceil(numel / 4096) <= 1,048,576 pieces
 * (4.29e9 elements when tensors are large); beyond either SELSYNC_ERR_TOO_LARGE is returned and
 * nothing is enqueued.  Other errors: INVALID_ARG, SHAPE_MISMATCH, DTYPE, NOT_DEVICE_MEM, HIP.
 * The result is deterministic (fixed slot per piece, fixed order of every sum) and differs from
 * selsync_track_grad_change's norm only by the grouping of the fp64 sum (about 1e-15 relative).
 * All calls on one GPU share the array: calls that may overlap in time on one GPU (different
 * streams, different threads) race and must be serialised by the caller.  Nothing in the array
 * needs clearing between calls (a call writes every slot it reads).
 * The first call on a GPU looks up the array's device address, and, as the first launch of any
 * kernel of a library does, makes the runtime load the library's device image there: a caller that
 * must not trigger that inside a capture or a timed loop makes one call beforehand.
 */
int32_t selsync_grad_norm_sq_noalloc(const selsync_tensor_list *grads, int32_t num_workers, float grad_scale,
                                     double *norm_sq_out, void *stream);

/* ---- data partitioning (Sec. III-D; the step before the hot path, Alg. 1 line 6) ------------ */

/*
 * Reading order of worker `worker` over `num_samples` samples split into num_workers
 * contiguous chunks DP0..DP(N-1) (the first num_samples % N chunks hold one sample more).
 *   scheme 0, default partitioning (DefDP): only the worker's own chunk, in order;
 *   scheme 1, SelSync partitioning (SelDP): all chunks as a circular queue whose head is
 *             rotated to the worker's own chunk: DPn, DP(n+1), ..., DP(n-1).
 * Writes min(*count, capacity) sample indices to `out` (HOST int64 array, may be NULL to only
 * query) and the length of the order to *count.  Pure host code, no GPU needed.
 */
int32_t selsync_partition_order(int64_t num_samples, int32_t num_workers, int32_t worker, int32_t scheme,
                                int64_t capacity, int64_t *out, int64_t *count);

/* The same order written into a DEVICE int64 array by a kernel on `stream` (for data pipelines
 * that gather samples on the GPU).  *count is a HOST output. */
int32_t selsync_partition_order_device(int64_t num_samples, int32_t num_workers, int32_t worker, int32_t scheme,
                                       int64_t capacity, int64_t *out_device, int64_t *count, void *stream);

/* ---- observability ---------------------------------------------------------------- */

/* Blocking fetch of the last step's device-side results (same outputs as tracking). */
int32_t selsync_read_decision(selsync_ctx *ctx, void *stream, double *norm_sq_out, double *delta_out,
                              int32_t *flags_out, int32_t *sync_out);

/*
 * Per-tensor squared gradient norms ||grad_scale*g_{k,t}||^2 of the LAST tracking pass
 * (selsync_track_grad_change or selsync_step) enqueued with this plan, summed from the same
 * per-chunk partials as the whole-model norm (Sec. II-E motivates per-layer gradient
 * statistics).  out: HOST array of num_workers * num_tensors doubles, index k*T + t.
 * Blocking.  SELSYNC_ERR_STATE if no tracking pass has run on the plan.
 */
int32_t selsync_read_tensor_norms(selsync_ctx *ctx, selsync_plan *plan, void *stream, double *out);

/* Blocking fetch of the cumulative counters (Eq. 4). */
int32_t selsync_get_stats(selsync_ctx *ctx, void *stream, selsync_stats *out);

/*
 * Checkpoint / resume of the tracker: windows, previous smoothed values, counters, the last
 * decision, delta (the device's and the host's copy) and the automatic first-step marker as one
 * opaque blob in HOST memory (tensors are the caller's to save).  A blob can only be restored
 * into a context with the same num_workers, window and alpha; restoring replaces that context's
 * delta by the blob's.  Both calls block on `stream`.
 */
int32_t selsync_tracker_state_size(const selsync_ctx *ctx, int64_t *bytes);
int32_t selsync_tracker_get_state(selsync_ctx *ctx, void *stream, void *buf, int64_t bytes);
int32_t selsync_tracker_set_state(selsync_ctx *ctx, void *stream, const void *buf, int64_t bytes);

/*
 * Per-kernel timing with HIP events recorded on the caller's stream around every
 * launch.  enable != 0 starts collecting (up to max_launches launches per kernel kind,
 * further launches are not timed); enable == 0 stops.  kind: 0 = streaming
 * update/norm kernel, 1 = tracker kernel, 2 = aggregation kernel.  The summary waits
 * for the recorded events, returns count and summed milliseconds, and clears them.
 */
int32_t selsync_profile_enable(selsync_ctx *ctx, int32_t enable, int32_t max_launches);
/* Which launches are timed: bit k of kind_mask selects kernel kind k (default 7 = all), and
 * only every stride-th launch of a selected kind is bracketed (default 1).  Event records
 * cost a few microseconds of stream time each, so a sparse setting keeps a timed loop honest. */
int32_t selsync_profile_config(selsync_ctx *ctx, int32_t kind_mask, int32_t stride);
int32_t selsync_profile_summary(selsync_ctx *ctx, int32_t kind, int64_t *count, double *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* SELSYNC_H */
