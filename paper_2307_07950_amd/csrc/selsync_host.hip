// Host side of the SelSync C ABI: contexts, plans (validation + chunk tables),
// per-step entry points and observability.  Every step of the path runs in the
// kernels of selsync_kernels.hip; this file only validates, builds tables once at
// plan time, and enqueues launches on the caller's stream.
#include "../../include/selsync.h"
#include "selsync_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <climits>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <vector>

using namespace selsync;

namespace {

constexpr int kDefaultChunkElems = kChunkGranule;   // one 128-bit access per lane and stream: a one-shot grid
constexpr int kDefaultGaChunkElems = 4096;   // few waves: on "local" decisions this launch only reads the decision
constexpr int kMaxWorkers = 1024;
constexpr int kSegChunks = 2048;          // chunks per segment of the intermediate reduction
constexpr int kDirectChunkLimit = 16384;  // up to this many chunks the tracker sums them directly
constexpr int kMaxWindow = 65536;

struct ProfRec {
    hipEvent_t start, stop;
};

// Address range of one bound tensor (for the overlap check).
struct Interval {
    uintptr_t lo, hi;
    bool written;
};

}  // namespace

struct selsync_ctx {
    selsync_config cfg;
    int device = 0;
    selsync_tuning tuning{0, -1, 0, 0};
    // device state: one allocation, sub-pointers in td
    void *d_state = nullptr;
    size_t state_bytes = 0;        // size of the d_state allocation
    size_t out_bytes = 0;          // bytes of the DecisionHeader block incl. the K-arrays
    TrackerDev td{};
    void *h_out = nullptr;         // pinned mirror of the decision block
    int64_t local_steps = 0;       // local updates enqueued since create/reset (automatic first-step)
    bool tracked = false;          // a tracking pass has been enqueued since create/reset (a decision exists)
    double tracked_delta = -1.0;   // threshold in force (host view) when the last tracking pass was enqueued;
                                   // only ever used to pick a launch SHAPE, never to decide whether to aggregate
    int live_plans = 0;
    std::string err;
    // profiling
    bool prof_on = false;
    int prof_cap = 0;
    std::vector<ProfRec> prof_pool[3];
    int prof_used[3] = {0, 0, 0};
    int64_t prof_seen[3] = {0, 0, 0};   // launches seen per kind since enable
    int prof_mask = 7;                  // bit k: time kernels of kind k
    int prof_stride = 1;                // time every prof_stride-th launch of a kind
};

struct selsync_plan {
    selsync_ctx *ctx = nullptr;
    int K = 0, T = 0;
    int64_t P = 0;
    bool mixed = false;
    bool has_grads = false;
    bool has_momenta = false;      // false with has_grads: momentum-free plan (plain SGD only)
    int n_upd_chunks = 0, n_agg_chunks = 0, n_ga_chunks = 0;
    void *d_blob = nullptr;        // all tables in one allocation
    TensorRec *d_recs = nullptr;
    StreamTable tab{};             // chunk table of the streaming kernels and its geometry
    int32_t *d_chunk_begin = nullptr;
    // intermediate reduction level (used when there are many chunks)
    int n_segs = 0;
    int2 *d_segs = nullptr;
    double *d_seg_sums = nullptr;
    int32_t *d_seg_begin = nullptr;
    // per-tensor norms (observability): chunk range of every (worker, tensor) pair
    int32_t *d_tensor_chunk_begin = nullptr;
    double *d_tensor_norms = nullptr;
    bool partials_valid = false;     // a tracking pass has been enqueued on this plan
    bool partials_from_sync = false; // ... and the last one was the one-pass synchronous step (its own partial array)
    // one-pass synchronous step: worker k's piece p is "chunk" k * t_fine.nslots + p of a partial array
    // striped with per = K * t_fine.per8 (see chunk_slot), and the reduction tables over those chunk numbers
    double *d_sync_partials = nullptr;
    int sync_per = 0;
    int32_t *d_sync_begin = nullptr;         // [K+1] worker k's partials
    int n_sync_segs = 0;
    int2 *d_sync_segs = nullptr;
    double *d_sync_seg_sums = nullptr;
    int32_t *d_sync_seg_begin = nullptr;     // [K+1]
    int32_t *d_sync_tensor_begin = nullptr;  // [K*T+1] partial range of every (worker, tensor) pair
    std::vector<TensorRec> h_recs;   // host copy (re-uploaded when second-moment buffers are bound)
    std::vector<int64_t> numel;      // per-tensor element counts
    std::vector<Interval> ivals;     // every bound buffer (checked again when more buffers are bound)
    bool has_second_moment = false;
    AggTable t_agg{};                     // pieces for aggregation launches that follow the device-side decision
    AggTable t_fine{};                    // 256-element pieces, striped by XCD: for launches that are expected to work
    AggTable t_ga{};                      // pieces of the decision-following gradient-aggregation launch
    AggTables agg{};
    float **d_agg_v = nullptr;            // device table behind agg.v (written when second moments are bound)
    bool nontemporal = true;              // streaming (non-temporal) loads and stores

    selsync_plan() = default;
    selsync_plan(const selsync_plan &) = delete;
    selsync_plan &operator=(const selsync_plan &) = delete;
    ~selsync_plan()
    {
        if (d_blob)
            (void)hipFree(d_blob);
    }
};

namespace {

int32_t fail(selsync_ctx *ctx, int32_t code, const char *fmt, ...)
{
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        ctx->err = buf;
    }
    return code;
}

#define HIP_TRY(ctx, expr)                                                                        \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess)                                                                     \
            return fail((ctx), e_ == hipErrorOutOfMemory ? SELSYNC_ERR_OOM : SELSYNC_ERR_HIP,     \
                        "%s failed: %s", #expr, hipGetErrorString(e_));                           \
    } while (0)

// Nothing may throw across the C boundary: host-side containers can (std::bad_alloc).
template <typename F>
int32_t guarded(selsync_ctx *ctx, F &&body)
{
    try {
        return body();
    } catch (const std::bad_alloc &) {
        return fail(ctx, SELSYNC_ERR_OOM, "out of host memory");
    } catch (...) {
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "unexpected internal error");
    }
}

int32_t check_device(selsync_ctx *ctx)
{
    int dev = -1;
    HIP_TRY(ctx, hipGetDevice(&dev));
    if (dev != ctx->device)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "current HIP device %d is not the context's device %d", dev,
                    ctx->device);
    return SELSYNC_OK;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

size_t dtype_size(int32_t dt) { return dt == SELSYNC_BF16 ? 2 : 4; }

// Profiling brackets around one launch.
struct ProfScope {
    selsync_ctx *ctx;
    int kind;
    hipStream_t s;
    ProfRec *rec = nullptr;
    ProfScope(selsync_ctx *c, int k, hipStream_t st) : ctx(c), kind(k), s(st)
    {
        if (ctx->prof_on && ((ctx->prof_mask >> kind) & 1)) {
            const bool pick = (ctx->prof_seen[kind]++ % ctx->prof_stride) == 0;
            if (pick && ctx->prof_used[kind] < ctx->prof_cap) {
                rec = &ctx->prof_pool[kind][ctx->prof_used[kind]++];
                (void)hipEventRecord(rec->start, s);
            }
        }
    }
    ~ProfScope()
    {
        if (rec)
            (void)hipEventRecord(rec->stop, s);
    }
};

// Validate one [K] array of lists against the reference shape; collect intervals.
int32_t check_lists(selsync_ctx *ctx, const char *what, const selsync_tensor_list *lists, int K, int T,
                    const std::vector<int64_t> &numel, int32_t want_dtype, bool written,
                    std::vector<Interval> &ivals)
{
    for (int k = 0; k < K; ++k) {
        const selsync_tensor_list &L = lists[k];
        if (L.count != T)
            return fail(ctx, SELSYNC_ERR_SHAPE_MISMATCH, "%s[%d] has %d tensors, expected %d", what, k, L.count, T);
        if (T > 0 && L.tensors == nullptr)
            return fail(ctx, SELSYNC_ERR_INVALID_ARG, "%s[%d].tensors is NULL", what, k);
        for (int t = 0; t < T; ++t) {
            const selsync_tensor &x = L.tensors[t];
            if (x.numel != numel[t])
                return fail(ctx, SELSYNC_ERR_SHAPE_MISMATCH, "%s[%d] tensor %d has %lld elements, expected %lld",
                            what, k, t, (long long)x.numel, (long long)numel[t]);
            if (x.dtype != SELSYNC_F32 && x.dtype != SELSYNC_BF16)
                return fail(ctx, SELSYNC_ERR_DTYPE, "%s[%d] tensor %d has unknown dtype %d", what, k, t, x.dtype);
            if (x.dtype != want_dtype)
                return fail(ctx, SELSYNC_ERR_DTYPE, "%s[%d] tensor %d has dtype %d, expected %d", what, k, t,
                            x.dtype, want_dtype);
            if (x.numel == 0)
                continue;
            if (x.data == nullptr)
                return fail(ctx, SELSYNC_ERR_INVALID_ARG, "%s[%d] tensor %d has NULL data", what, k, t);
            const size_t es = dtype_size(x.dtype);
            if (reinterpret_cast<uintptr_t>(x.data) % es != 0)
                return fail(ctx, SELSYNC_ERR_INVALID_ARG, "%s[%d] tensor %d is not aligned to its element size",
                            what, k, t);
            hipPointerAttribute_t attr;
            hipError_t e = hipPointerGetAttributes(&attr, x.data);
            if (e != hipSuccess) {
                (void)hipGetLastError();
                return fail(ctx, SELSYNC_ERR_NOT_DEVICE_MEM, "%s[%d] tensor %d: pointer %p is not known to HIP",
                            what, k, t, x.data);
            }
            if (attr.type != hipMemoryTypeDevice || attr.device != ctx->device)
                return fail(ctx, SELSYNC_ERR_NOT_DEVICE_MEM,
                            "%s[%d] tensor %d: pointer %p is not device memory of GPU %d", what, k, t, x.data,
                            ctx->device);
            const uintptr_t lo = reinterpret_cast<uintptr_t>(x.data);
            ivals.push_back({lo, lo + (uintptr_t)x.numel * es, written});
        }
    }
    return SELSYNC_OK;
}

int32_t check_overlap(selsync_ctx *ctx, std::vector<Interval> &iv)
{
    // Sorted sweep.  Read-only buffers may overlap each other (the same gradient may be
    // bound to several workers); a written buffer may overlap nothing.
    std::sort(iv.begin(), iv.end(), [](const Interval &a, const Interval &b) { return a.lo < b.lo; });
    uintptr_t max_hi = 0;     // furthest end of any interval seen so far
    uintptr_t max_hi_w = 0;   // furthest end of any written interval seen so far
    for (size_t i = 0; i < iv.size(); ++i) {
        if (iv[i].lo < max_hi_w)
            return fail(ctx, SELSYNC_ERR_INVALID_ARG, "a tensor buffer overlaps a written buffer near %p",
                        (void *)iv[i].lo);
        if (iv[i].written && iv[i].lo < max_hi)
            return fail(ctx, SELSYNC_ERR_INVALID_ARG, "a written tensor buffer overlaps another buffer near %p",
                        (void *)iv[i].lo);
        max_hi = std::max(max_hi, iv[i].hi);
        if (iv[i].written)
            max_hi_w = std::max(max_hi_w, iv[i].hi);
    }
    return SELSYNC_OK;
}

// Phase of a stream: element index (mod 4) of its first element relative to vector alignment
// (16 bytes for fp32 streams, 8 bytes for bf16 streams).  Streams with equal phase become
// vector-aligned together after peeling (4 - phase) % 4 elements.
int stream_phase(const void *p, size_t elem_size)
{
    return (int)((reinterpret_cast<uintptr_t>(p) / elem_size) & 3u);
}

uint32_t head_bits(int phase) { return (uint32_t)((4 - phase) & 3) << kChunkHeadShift; }

// The chunking rule of the multi-tensor tables.  A tensor whose first element lies `lead`
// elements past a chunk-size-aligned address (0 <= lead < chunk) is cut where its ADDRESSES
// cross multiples of the chunk size: a first piece of up to chunk - lead elements, full
// pieces, one shorter last piece.  Piece j covers elements [j*chunk - lead, (j+1)*chunk - lead)
// clipped to [0, numel); empty tensors give none.  With lead = 0 this is plain cutting
// from element 0.  A wavefront's 1 KiB accesses then never straddle cache lines or DRAM
// interleave boundaries, wherever in an arena the tensor starts.
template <typename Emit>
void split_tensor(int64_t numel, int chunk, int lead, Emit emit)
{
    if (numel <= 0)
        return;
    const int64_t vend = (int64_t)lead + numel;
    for (int64_t j = 0; j * chunk < vend; ++j) {
        const int64_t b = std::max<int64_t>(j * chunk, lead) - lead;
        const int64_t e = std::min<int64_t>((j + 1) * chunk, vend) - lead;
        emit(b, e - b, j);
    }
}

// One stream of a chunk (address, element size, bytes it moves per element).
struct StreamRef {
    const void *p;
    int elem_size;
    int weight;
};

// The lead (see split_tensor) that aligns the most traffic: every stream proposes
// (address / element size) mod chunk; the proposal backed by the most bytes wins, the
// first stream breaking ties.
int vote_lead(const std::vector<StreamRef> &streams, int chunk)
{
    int best = 0, best_w = -1;
    for (size_t i = 0; i < streams.size(); ++i) {
        if (!streams[i].p)
            continue;
        const int li = (int)((reinterpret_cast<uintptr_t>(streams[i].p) / (uintptr_t)streams[i].elem_size) % (uintptr_t)chunk);
        int w = 0;
        for (size_t j = 0; j < streams.size(); ++j)
            if (streams[j].p &&
                (int)((reinterpret_cast<uintptr_t>(streams[j].p) / (uintptr_t)streams[j].elem_size) % (uintptr_t)chunk) == li)
                w += streams[j].weight;
        if (w > best_w) {
            best_w = w;
            best = li;
        }
    }
    return best;
}

// Elements per aggregation chunk: 256 threads x 4 vectors of 4 elements.  Each thread keeps
// K*4 128-bit loads in flight; the working launch streams within two or three points of the finest
// pieces (71 % against 73 % of peak at K = 4), and the launch has 16 times fewer workgroups than one
// of single-wavefront pieces, which is what counts on local steps, where it only reads the decision
// and exits (about 0.2 ns per dispatched workgroup: 8 us against 110 us).
int default_agg_chunk(int) { return 4 * kAggTileElems; }

int effective_chunk(const selsync_ctx *ctx)
{
    return ctx->tuning.chunk_elems > 0 ? ctx->tuning.chunk_elems : kDefaultChunkElems;
}

int32_t fetch_decision(selsync_ctx *ctx, hipStream_t s, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                       int32_t *sync_out, DecisionHeader *hdr_out)
{
    HIP_TRY(ctx, hipMemcpyAsync(ctx->h_out, ctx->td.out, ctx->out_bytes, hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipStreamSynchronize(s));
    const int K = ctx->cfg.num_workers;
    const char *base = static_cast<const char *>(ctx->h_out);
    const DecisionHeader *hdr = reinterpret_cast<const DecisionHeader *>(base);
    const double *nrm = reinterpret_cast<const double *>(base + sizeof(DecisionHeader));
    const double *dlt = nrm + K;
    const int32_t *flg = reinterpret_cast<const int32_t *>(dlt + 2 * K);
    if (norm_sq_out)
        std::memcpy(norm_sq_out, nrm, sizeof(double) * K);
    if (delta_out)
        std::memcpy(delta_out, dlt, sizeof(double) * K);
    if (flags_out)
        std::memcpy(flags_out, flg, sizeof(int32_t) * K);
    if (sync_out)
        *sync_out = hdr->sync;
    if (hdr_out)
        *hdr_out = *hdr;
    return hdr->nonfinite_now ? SELSYNC_WARN_NONFINITE : SELSYNC_OK;
}

int32_t resolve_sgd(selsync_ctx *ctx, const selsync_plan *plan, const selsync_sgd *sgd, SgdArgs *out)
{
    if (!sgd)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "sgd is NULL");
    if (sgd->first_step < -1 || sgd->first_step > 1)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "sgd.first_step must be -1, 0 or 1");
    if (sgd->nesterov != 0 && sgd->nesterov != 1)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "sgd.nesterov must be 0 or 1");
    if (sgd->nesterov && !(sgd->momentum > 0.f))
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "sgd.nesterov needs momentum > 0");
    if (!plan->has_momenta && (sgd->momentum != 0.f || sgd->nesterov))
        return fail(ctx, SELSYNC_ERR_INVALID_ARG,
                    "the plan has no momentum buffers: momentum must be 0 and nesterov 0");
    out->nesterov = sgd->nesterov;
    out->lr = sgd->lr;
    out->mu = sgd->momentum;
    out->wd = sgd->weight_decay;
    out->gs = sgd->grad_scale;
    out->first = sgd->first_step < 0 ? (ctx->local_steps == 0 ? 1 : 0) : sgd->first_step;
    return SELSYNC_OK;
}

// a1 final passes + a2: (optional) segment reduction, then the single-workgroup tracker.
int32_t enqueue_track(selsync_ctx *ctx, selsync_plan *plan, hipStream_t s, bool from_sync = false)
{
    plan->partials_valid = true;
    plan->partials_from_sync = from_sync;
    ctx->tracked = true;
    ctx->tracked_delta = ctx->cfg.delta;
    ProfScope p(ctx, 1, s);
    if (from_sync) {
        // partials of the one-pass synchronous step (their own striped array)
        if (plan->n_sync_segs > 0) {
            HIP_TRY(ctx, launch_reduce(plan->d_sync_partials, plan->sync_per, plan->d_sync_segs, plan->n_sync_segs,
                                       plan->d_sync_seg_sums, s));
            HIP_TRY(ctx, launch_track(ctx->td, plan->d_sync_seg_sums, 0, plan->d_sync_seg_begin, s));
        } else {
            HIP_TRY(ctx, launch_track(ctx->td, plan->d_sync_partials, plan->sync_per, plan->d_sync_begin, s));
        }
        return SELSYNC_OK;
    }
    if (plan->n_segs > 0) {
        HIP_TRY(ctx, launch_reduce(plan->tab.partials, plan->tab.per, plan->d_segs, plan->n_segs, plan->d_seg_sums, s));
        HIP_TRY(ctx, launch_track(ctx->td, plan->d_seg_sums, 0, plan->d_seg_begin, s));
    } else {
        HIP_TRY(ctx, launch_track(ctx->td, plan->tab.partials, plan->tab.per, plan->d_chunk_begin, s));
    }
    return SELSYNC_OK;
}

// True when the last decision enqueued on this context was taken under a threshold of 0, under which
// every tracked step decides "sync" (Delta >= 0 always holds, +inf included).  A hint for the launch
// shape only: launches still follow the device-side decision word.
bool expect_sync(const selsync_ctx *ctx) { return ctx->tracked && ctx->tracked_delta == 0.0; }

int32_t check_plan(selsync_ctx *ctx, selsync_plan *plan, bool need_grads, bool need_momenta = false)
{
    if (!ctx)
        return SELSYNC_ERR_INVALID_ARG;
    if (!plan)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "plan is NULL");
    if (plan->ctx != ctx)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "plan belongs to a different context");
    if (need_grads && !plan->has_grads)
        return fail(ctx, SELSYNC_ERR_STATE, "plan was created without gradients");
    if (need_momenta && !plan->has_momenta)
        return fail(ctx, SELSYNC_ERR_STATE, "plan was created without momentum buffers");
    return check_device(ctx);
}

}  // namespace

// =============================================================================== lifecycle

extern "C" const char *selsync_status_string(int32_t status)
{
    switch (status) {
    case SELSYNC_OK: return "SELSYNC_OK";
    case SELSYNC_ERR_INVALID_ARG: return "SELSYNC_ERR_INVALID_ARG";
    case SELSYNC_ERR_SHAPE_MISMATCH: return "SELSYNC_ERR_SHAPE_MISMATCH";
    case SELSYNC_ERR_DTYPE: return "SELSYNC_ERR_DTYPE";
    case SELSYNC_ERR_OOM: return "SELSYNC_ERR_OOM";
    case SELSYNC_ERR_HIP: return "SELSYNC_ERR_HIP";
    case SELSYNC_ERR_NOT_DEVICE_MEM: return "SELSYNC_ERR_NOT_DEVICE_MEM";
    case SELSYNC_ERR_STATE: return "SELSYNC_ERR_STATE";
    case SELSYNC_ERR_TOO_LARGE: return "SELSYNC_ERR_TOO_LARGE";
    case SELSYNC_WARN_NONFINITE: return "SELSYNC_WARN_NONFINITE";
    default: return "SELSYNC_UNKNOWN_STATUS";
    }
}

extern "C" const char *selsync_last_error(const selsync_ctx *ctx) { return ctx ? ctx->err.c_str() : "context is NULL"; }

extern "C" int32_t selsync_create(const selsync_config *cfg, selsync_ctx **out)
{
    if (!out)
        return SELSYNC_ERR_INVALID_ARG;
    *out = nullptr;
    if (!cfg)
        return SELSYNC_ERR_INVALID_ARG;
    if (cfg->num_workers < 1 || cfg->num_workers > kMaxWorkers)
        return SELSYNC_ERR_INVALID_ARG;
    if (cfg->window < 0 || cfg->window > kMaxWindow)
        return SELSYNC_ERR_INVALID_ARG;
    if (!(cfg->delta >= 0.0))   // rejects negatives and NaN, accepts +inf
        return SELSYNC_ERR_INVALID_ARG;
    if (cfg->alpha > 1.0 || cfg->alpha != cfg->alpha)
        return SELSYNC_ERR_INVALID_ARG;

    selsync_ctx *ctx = new (std::nothrow) selsync_ctx();
    if (!ctx)
        return SELSYNC_ERR_OOM;
    ctx->cfg = *cfg;
    if (ctx->cfg.window == 0)
        ctx->cfg.window = 25;
    if (ctx->cfg.alpha <= 0.0)
        ctx->cfg.alpha = (double)ctx->cfg.num_workers / 100.0;
    if (ctx->cfg.alpha > 1.0)
        ctx->cfg.alpha = 1.0;
    const int K = ctx->cfg.num_workers, W = ctx->cfg.window;

    auto bail = [&](int32_t code) {
        if (ctx->d_state)
            (void)hipFree(ctx->d_state);
        if (ctx->h_out)
            (void)hipHostFree(ctx->h_out);
        delete ctx;
        return code;
    };

    if (hipGetDevice(&ctx->device) != hipSuccess)
        return bail(SELSYNC_ERR_HIP);

    // layout of the single state allocation
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    ctx->out_bytes = sizeof(DecisionHeader) + sizeof(double) * 3 * K + sizeof(int32_t) * K;
    const size_t o_out = take(ctx->out_bytes);
    const size_t o_hist = take(sizeof(double) * (size_t)K * W);
    const size_t o_len = take(sizeof(int32_t) * K);
    const size_t o_head = take(sizeof(int32_t) * K);
    const size_t o_sprev = take(sizeof(double) * K);
    const size_t o_hasprev = take(sizeof(int32_t) * K);
    const size_t o_weights = take(sizeof(double) * W);
    const size_t o_thr = take(sizeof(double));
    ctx->state_bytes = off;
    hipError_t e = hipMalloc(&ctx->d_state, off);
    if (e != hipSuccess)
        return bail(e == hipErrorOutOfMemory ? SELSYNC_ERR_OOM : SELSYNC_ERR_HIP);
    e = hipHostMalloc(&ctx->h_out, ctx->out_bytes, hipHostMallocDefault);
    if (e != hipSuccess)
        return bail(e == hipErrorOutOfMemory ? SELSYNC_ERR_OOM : SELSYNC_ERR_HIP);

    char *b = static_cast<char *>(ctx->d_state);
    TrackerDev &td = ctx->td;
    td.out = reinterpret_cast<DecisionHeader *>(b + o_out);
    td.out_norm_sq = reinterpret_cast<double *>(b + o_out + sizeof(DecisionHeader));
    td.out_delta = td.out_norm_sq + K;
    td.out_smoothed = td.out_delta + K;
    td.out_flags = reinterpret_cast<int32_t *>(td.out_smoothed + K);
    td.hist = reinterpret_cast<double *>(b + o_hist);
    td.len = reinterpret_cast<int32_t *>(b + o_len);
    td.head = reinterpret_cast<int32_t *>(b + o_head);
    td.s_prev = reinterpret_cast<double *>(b + o_sprev);
    td.has_prev = reinterpret_cast<int32_t *>(b + o_hasprev);
    td.weights = reinterpret_cast<const double *>(b + o_weights);
    td.delta_thr = reinterpret_cast<double *>(b + o_thr);
    td.K = K;
    td.window = W;

    // EWMA weights: a sample of age j weighs (1-alpha)^j (Sec. III-A smoothing)
    std::vector<double> wts(W);
    for (int j = 0; j < W; ++j)
        wts[j] = std::pow(1.0 - ctx->cfg.alpha, (double)j);
    if (hipMemcpy(b + o_weights, wts.data(), sizeof(double) * W, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(b + o_thr, &ctx->cfg.delta, sizeof(double), hipMemcpyHostToDevice) != hipSuccess ||
        launch_reset(td, nullptr) != hipSuccess || hipDeviceSynchronize() != hipSuccess)
        return bail(SELSYNC_ERR_HIP);

    *out = ctx;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_destroy(selsync_ctx *ctx)
{
    if (!ctx)
        return SELSYNC_OK;
    if (ctx->live_plans != 0)
        return fail(ctx, SELSYNC_ERR_STATE, "%d plan(s) still alive", ctx->live_plans);
    (void)hipDeviceSynchronize();
    for (int k = 0; k < 3; ++k)
        for (auto &r : ctx->prof_pool[k]) {
            (void)hipEventDestroy(r.start);
            (void)hipEventDestroy(r.stop);
        }
    if (ctx->d_state)
        (void)hipFree(ctx->d_state);
    if (ctx->h_out)
        (void)hipHostFree(ctx->h_out);
    delete ctx;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_reset(selsync_ctx *ctx, void *stream)
{
    if (!ctx)
        return SELSYNC_ERR_INVALID_ARG;
    int32_t rc = check_device(ctx);
    if (rc)
        return rc;
    HIP_TRY(ctx, launch_reset(ctx->td, static_cast<hipStream_t>(stream)));
    ctx->local_steps = 0;
    ctx->tracked = false;
    ctx->tracked_delta = -1.0;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_set_delta(selsync_ctx *ctx, double delta, void *stream)
{
    if (!ctx)
        return SELSYNC_ERR_INVALID_ARG;
    if (!(delta >= 0.0))
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "delta must be >= 0");
    int32_t rc = check_device(ctx);
    if (rc)
        return rc;
    HIP_TRY(ctx, launch_set_delta(ctx->td, delta, static_cast<hipStream_t>(stream)));
    ctx->cfg.delta = delta;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_set_tuning(selsync_ctx *ctx, const selsync_tuning *t)
{
    if (!ctx || !t)
        return SELSYNC_ERR_INVALID_ARG;
    const struct { const char *name; int32_t v; } sizes[] = {
        {"chunk_elems", t->chunk_elems}, {"agg_chunk_elems", t->agg_chunk_elems}, {"ga_chunk_elems", t->ga_chunk_elems}};
    for (const auto &z : sizes)
        if (z.v > 0 && (z.v % kChunkGranule != 0 || z.v > (1 << 24)))
            return fail(ctx, SELSYNC_ERR_INVALID_ARG, "%s must be a multiple of %d and <= 2^24", z.name, kChunkGranule);
    ctx->tuning = *t;
    return SELSYNC_OK;
}

// =============================================================================== plan

namespace {
int32_t plan_create_impl(selsync_ctx *ctx, const selsync_tensor_list *grads, const selsync_tensor_list *params,
                         const selsync_tensor_list *momenta, const selsync_tensor_list *master,
                         const selsync_tensor_list *global, const selsync_tensor_list *global_lowp, selsync_plan **out);
}

extern "C" int32_t selsync_plan_create(selsync_ctx *ctx, const selsync_tensor_list *grads,
                                       const selsync_tensor_list *params, const selsync_tensor_list *momenta,
                                       const selsync_tensor_list *master, const selsync_tensor_list *global,
                                       const selsync_tensor_list *global_lowp, selsync_plan **out)
{
    if (!ctx)
        return SELSYNC_ERR_INVALID_ARG;
    if (!out)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    return guarded(ctx, [&] { return plan_create_impl(ctx, grads, params, momenta, master, global, global_lowp, out); });
}

namespace {
int32_t plan_create_impl(selsync_ctx *ctx, const selsync_tensor_list *grads, const selsync_tensor_list *params,
                         const selsync_tensor_list *momenta, const selsync_tensor_list *master,
                         const selsync_tensor_list *global, const selsync_tensor_list *global_lowp, selsync_plan **out)
{
    int32_t rc = check_device(ctx);
    if (rc)
        return rc;
    if (!params || !global)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "params and global are required");
    if (momenta != nullptr && grads == nullptr)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "momenta given without grads");
    const bool mixed = master != nullptr;
    if (mixed != (global_lowp != nullptr))
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "master and global_lowp must be given together (mixed mode)");

    const int K = ctx->cfg.num_workers;
    const int T = params[0].count;
    if (T < 0)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "negative tensor count");
    if (T > 0 && params[0].tensors == nullptr)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "params[0].tensors is NULL");
    std::vector<int64_t> numel(T);
    int64_t P = 0;
    for (int t = 0; t < T; ++t) {
        numel[t] = params[0].tensors[t].numel;
        if (numel[t] < 0)
            return fail(ctx, SELSYNC_ERR_INVALID_ARG, "tensor %d has negative numel", t);
        P += numel[t];
    }

    std::vector<Interval> ivals;
    ivals.reserve((size_t)T * (4 * K + 2));
    const int32_t lowp = SELSYNC_BF16;
    if ((rc = check_lists(ctx, "params", params, K, T, numel, mixed ? lowp : SELSYNC_F32, true, ivals)))
        return rc;
    if (grads) {
        if ((rc = check_lists(ctx, "grads", grads, K, T, numel, mixed ? lowp : SELSYNC_F32, false, ivals)))
            return rc;
        if (momenta && (rc = check_lists(ctx, "momenta", momenta, K, T, numel, SELSYNC_F32, true, ivals)))
            return rc;
    }
    if (mixed) {
        if ((rc = check_lists(ctx, "master", master, K, T, numel, SELSYNC_F32, true, ivals)))
            return rc;
        if ((rc = check_lists(ctx, "global_lowp", global_lowp, 1, T, numel, lowp, true, ivals)))
            return rc;
    }
    if ((rc = check_lists(ctx, "global", global, 1, T, numel, SELSYNC_F32, true, ivals)))
        return rc;
    if ((rc = check_overlap(ctx, ivals)))
        return rc;

    const int chunk = effective_chunk(ctx);
    const int agg_chunk = ctx->tuning.agg_chunk_elems > 0 ? ctx->tuning.agg_chunk_elems : default_agg_chunk(K);
    const int ga_chunk = ctx->tuning.ga_chunk_elems > 0 ? ctx->tuning.ga_chunk_elems : kDefaultGaChunkElems;
    // Streaming (non-temporal) accesses pay off once the working set is far beyond the last-level
    // cache (measured: +11 % at 435 MB); below roughly half its 256 MB plain accesses are 3-6 % faster.
    const int64_t working_set = (int64_t)K * P * 12;   // g, w, m: 12 bytes per parameter in either precision
    const int nt = ctx->tuning.nontemporal >= 0 ? ctx->tuning.nontemporal : (working_set >= (int64_t)128 << 20);

    // ---- host tables
    std::vector<TensorRec> recs;
    std::vector<ChunkRec> chunks;     // in chunk order: worker by worker, tensor by tensor
    std::vector<int32_t> chunk_begin(K + 1, 0);
    std::vector<int32_t> tensor_chunk_begin((size_t)K * T + 1, 0);
    if (grads) {
        recs.resize((size_t)K * T);
        for (int k = 0; k < K; ++k) {
            chunk_begin[k] = (int32_t)chunks.size();
            for (int t = 0; t < T; ++t) {
                TensorRec r{};
                r.g = grads[k].tensors[t].data;
                r.m = momenta ? static_cast<float *>(momenta[k].tensors[t].data) : nullptr;
                if (mixed) {
                    r.w = static_cast<float *>(master[k].tensors[t].data);
                    r.lowp = static_cast<uint16_t *>(params[k].tensors[t].data);
                } else {
                    r.w = static_cast<float *>(params[k].tensors[t].data);
                    r.lowp = nullptr;
                }
                tensor_chunk_begin[(size_t)k * T + t] = (int32_t)chunks.size();
                const int ph = stream_phase(r.w, 4);
                const bool al = stream_phase(r.g, mixed ? 2 : 4) == ph && (!r.m || stream_phase(r.m, 4) == ph) &&
                                (!mixed || stream_phase(r.lowp, 2) == ph);
                r.numel = numel[t];
                r.flags = al ? (kChunkAligned | head_bits(ph)) : 0u;
                // bytes per element: w and m are read and written, g is read, the bf16 copy written
                r.lead = (uint32_t)vote_lead({{r.w, 4, 8}, {r.m, 4, 8}, {r.g, mixed ? 2 : 4, mixed ? 2 : 4},
                                              {r.lowp, 2, 2}}, chunk);
                recs[(size_t)k * T + t] = r;
                split_tensor(numel[t], chunk, (int)r.lead, [&](int64_t, int64_t, int64_t j) {
                    ChunkRec c;
                    c.rec = (uint32_t)((size_t)k * T + t);
                    c.j = (uint32_t)j;
                    chunks.push_back(c);
                });
            }
        }
        chunk_begin[K] = (int32_t)chunks.size();
        tensor_chunk_begin[(size_t)K * T] = (int32_t)chunks.size();
    }
    if (chunks.size() > (size_t)INT32_MAX - 8 * kStripeGranule)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "model too large for one plan (%zu chunks)", chunks.size());

    // Slot order of the table (and of the partial sums): 8 stripes of `per` slots, padded with empty
    // slots; workgroup b of the streaming kernel works on stripe b % 8.
    const int nchunks = (int)chunks.size();
    const int per = nchunks > 0 ? (int)align_up((size_t)(nchunks + 7) / 8, kStripeGranule) : 0;
    const int nslots = 8 * per;
    std::vector<ChunkRec> slots((size_t)nslots, ChunkRec{kNoChunk, 0u});
    for (int c = 0; c < nchunks; ++c)
        slots[(size_t)chunk_slot(c, per)] = chunks[c];

    // With many chunks the per-chunk partials first collapse into fixed segments of
    // kSegChunks consecutive chunks (never crossing a worker boundary); the tracker kernel
    // then sums segment results.  Small models skip this level.
    std::vector<int2> segs;
    std::vector<int32_t> seg_begin(K + 1, 0);
    if (grads && chunks.size() > (size_t)kDirectChunkLimit) {
        for (int k = 0; k < K; ++k) {
            seg_begin[k] = (int32_t)segs.size();
            for (int32_t b0 = chunk_begin[k]; b0 < chunk_begin[k + 1]; b0 += kSegChunks)
                segs.push_back(make_int2(b0, std::min<int32_t>(b0 + kSegChunks, chunk_begin[k + 1])));
        }
        seg_begin[K] = (int32_t)segs.size();
    }

    std::vector<AggChunkRec> agg_chunks, agg_fine, ga_chunks;
    std::vector<float *> agg_w((size_t)T * K);
    std::vector<uint16_t *> agg_c(mixed ? (size_t)T * K : 0);
    std::vector<float *> agg_g(T);
    std::vector<uint16_t *> agg_gc(mixed ? T : 0);
    std::vector<const void *> agg_grad(grads ? (size_t)T * K : 0);
    std::vector<float *> agg_m(momenta ? (size_t)T * K : 0);
    for (int t = 0; t < T; ++t) {
        agg_g[t] = static_cast<float *>(global[0].tensors[t].data);
        const int ph = stream_phase(agg_g[t], 4);
        bool al = true;
        for (int k = 0; k < K; ++k) {
            if (mixed) {
                agg_w[(size_t)t * K + k] = static_cast<float *>(master[k].tensors[t].data);
                agg_c[(size_t)t * K + k] = static_cast<uint16_t *>(params[k].tensors[t].data);
                al = al && stream_phase(agg_c[(size_t)t * K + k], 2) == ph;
            } else {
                agg_w[(size_t)t * K + k] = static_cast<float *>(params[k].tensors[t].data);
            }
            al = al && stream_phase(agg_w[(size_t)t * K + k], 4) == ph;
        }
        bool al_grads = grads != nullptr;
        if (grads) {
            for (int k = 0; k < K; ++k) {
                agg_grad[(size_t)t * K + k] = grads[k].tensors[t].data;
                al_grads = al_grads && stream_phase(agg_grad[(size_t)t * K + k], mixed ? 2 : 4) == ph;
                if (momenta) {
                    agg_m[(size_t)t * K + k] = static_cast<float *>(momenta[k].tensors[t].data);
                    al_grads = al_grads && stream_phase(agg_m[(size_t)t * K + k], 4) == ph;
                }
            }
        }
        if (mixed) {
            agg_gc[t] = static_cast<uint16_t *>(global_lowp[0].tensors[t].data);
            al = al && stream_phase(agg_gc[t], 2) == ph;
        }
        // only a tensor's first piece can start off vector alignment: later pieces start on
        // chunk-size-aligned addresses of the streams that share the phase
        std::vector<StreamRef> refs;
        refs.push_back({agg_g[t], 4, 4});
        for (int k = 0; k < K; ++k)
            refs.push_back({agg_w[(size_t)t * K + k], 4, 8});
        split_tensor(numel[t], agg_chunk, vote_lead(refs, agg_chunk), [&](int64_t off, int64_t n, int64_t j) {
            AggChunkRec c;
            c.t = (uint32_t)t;
            c.n_flags = (uint32_t)n | (al ? (kChunkAligned | (j == 0 ? head_bits(ph) : 0u)) : 0u) |
                        (al_grads ? kChunkAlignedGrads : 0u);
            c.off = (uint64_t)off;
            agg_chunks.push_back(c);
        });
        split_tensor(numel[t], kChunkGranule, vote_lead(refs, kChunkGranule), [&](int64_t off, int64_t n, int64_t j) {
            AggChunkRec c;
            c.t = (uint32_t)t;
            c.n_flags = (uint32_t)n | (al ? (kChunkAligned | (j == 0 ? head_bits(ph) : 0u)) : 0u) |
                        (al_grads ? kChunkAlignedGrads : 0u);
            c.off = (uint64_t)off;
            agg_fine.push_back(c);
        });
        if (grads) {
            refs.clear();
            for (int k = 0; k < K; ++k) {
                refs.push_back({agg_w[(size_t)t * K + k], 4, 8});
                refs.push_back({momenta ? agg_m[(size_t)t * K + k] : nullptr, 4, 8});
                refs.push_back({agg_grad[(size_t)t * K + k], mixed ? 2 : 4, mixed ? 2 : 4});
            }
            split_tensor(numel[t], ga_chunk, vote_lead(refs, ga_chunk), [&](int64_t off, int64_t n, int64_t j) {
                AggChunkRec c;
                c.t = (uint32_t)t;
                c.n_flags = (uint32_t)n | (al ? (kChunkAligned | (j == 0 ? head_bits(ph) : 0u)) : 0u) |
                            (al_grads ? kChunkAlignedGrads : 0u);
                c.off = (uint64_t)off;
                ga_chunks.push_back(c);
            });
        }
    }
    if (agg_chunks.size() > (size_t)INT32_MAX || ga_chunks.size() > (size_t)INT32_MAX ||
        (agg_fine.size() + 8) * (size_t)std::max(K, 1) > (size_t)INT32_MAX)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "model too large for one plan");

    // The 256-element table is stored in 8 stripes (piece p in slot (p % 8) * per8 + p / 8, padded with empty
    // records): workgroup p of a launch runs on XCD p % 8, so each table line is fetched by one L2.
    const int np = (int)agg_fine.size();
    const int per8 = (np + 7) / 8;
    const int np_pad = 8 * per8;
    std::vector<AggChunkRec> fine_striped((size_t)np_pad, AggChunkRec{0u, 0u, 0u});
    for (int i = 0; i < np; ++i)
        fine_striped[(size_t)(i & 7) * per8 + (i >> 3)] = agg_fine[i];

    // Partial sums of the one-pass synchronous step: worker k's piece p is chunk k * np_pad + p of an array
    // striped like the streaming kernel's (per = K * per8).  Same two-level scheme on top: fixed segments of
    // kSegChunks consecutive chunks that never cross a worker boundary once there are many.
    std::vector<int32_t> sync_begin(K + 1, 0), sync_seg_begin(K + 1, 0), sync_tensor_begin((size_t)K * T + 1, 0);
    std::vector<int2> sync_segs;
    if (grads) {
        std::vector<int32_t> fine_begin(T + 1, 0);        // first piece of every tensor
        {
            int t_prev = 0;
            for (int i = 0; i < np; ++i)
                for (; t_prev <= (int)agg_fine[i].t; ++t_prev)
                    fine_begin[t_prev] = i;
            for (; t_prev <= T; ++t_prev)
                fine_begin[t_prev] = np;
        }
        // worker k's chunks are [k * np_pad, k * np_pad + np); the few padding chunks behind them are never
        // written and stay zero (they fall into the last tensor's range below, where they add nothing)
        for (int k = 0; k <= K; ++k)
            sync_begin[k] = k * np_pad;
        for (int k = 0; k < K; ++k)
            for (int t = 0; t < T; ++t)
                sync_tensor_begin[(size_t)k * T + t] = k * np_pad + fine_begin[t];
        sync_tensor_begin[(size_t)K * T] = K * np_pad;
        if ((size_t)K * np > (size_t)kDirectChunkLimit) {
            for (int k = 0; k < K; ++k) {
                sync_seg_begin[k] = (int32_t)sync_segs.size();
                for (int32_t b0 = k * np_pad; b0 < k * np_pad + np; b0 += kSegChunks)
                    sync_segs.push_back(make_int2(b0, std::min<int32_t>(b0 + kSegChunks, k * np_pad + np)));
            }
            sync_seg_begin[K] = (int32_t)sync_segs.size();
        }
    }

    std::unique_ptr<selsync_plan> plan(new selsync_plan());     // frees its device tables on any early exit
    plan->ctx = ctx;
    plan->K = K;
    plan->T = T;
    plan->P = P;
    plan->mixed = mixed;
    plan->has_grads = grads != nullptr;
    plan->has_momenta = momenta != nullptr;
    plan->h_recs = recs;
    plan->numel = numel;
    plan->ivals = ivals;
    plan->n_upd_chunks = nchunks;
    plan->n_agg_chunks = (int)agg_chunks.size();
    plan->n_ga_chunks = (int)ga_chunks.size();
    plan->nontemporal = nt != 0;

    // ---- one device allocation for every table
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + std::max<size_t>(bytes, 8), 256);
        return o;
    };
    const size_t o_recs = take(recs.size() * sizeof(TensorRec));
    const size_t o_chunks = take(slots.size() * sizeof(ChunkRec));
    const size_t o_begin = take(chunk_begin.size() * sizeof(int32_t));
    const size_t o_part = take(slots.size() * sizeof(double));
    const size_t o_segs = take(segs.size() * sizeof(int2));
    const size_t o_segsum = take(segs.size() * sizeof(double));
    const size_t o_segbegin = take(seg_begin.size() * sizeof(int32_t));
    const size_t o_tcb = take(tensor_chunk_begin.size() * sizeof(int32_t));
    const size_t o_tnorm = take((size_t)K * T * sizeof(double));
    const size_t o_aggc = take(agg_chunks.size() * sizeof(AggChunkRec));
    const size_t o_aggf = take(fine_striped.size() * sizeof(AggChunkRec));
    const size_t o_gac = take(ga_chunks.size() * sizeof(AggChunkRec));
    const size_t o_spart = take(grads ? (size_t)K * np_pad * sizeof(double) : 0);
    const size_t o_sbegin = take(sync_begin.size() * sizeof(int32_t));
    const size_t o_ssegs = take(sync_segs.size() * sizeof(int2));
    const size_t o_ssegsum = take(sync_segs.size() * sizeof(double));
    const size_t o_ssegbegin = take(sync_seg_begin.size() * sizeof(int32_t));
    const size_t o_stb = take(sync_tensor_begin.size() * sizeof(int32_t));
    const size_t o_aw = take(agg_w.size() * sizeof(float *));
    const size_t o_ac = take(agg_c.size() * sizeof(uint16_t *));
    const size_t o_ag = take(agg_g.size() * sizeof(float *));
    const size_t o_agc = take(agg_gc.size() * sizeof(uint16_t *));
    const size_t o_agrad = take(agg_grad.size() * sizeof(void *));
    const size_t o_am = take(agg_m.size() * sizeof(float *));
    const size_t o_av = take(agg_m.size() * sizeof(float *));     // second-moment table, filled when they are bound

    std::vector<char> blob(off, 0);
    auto put = [&](size_t o, const void *src, size_t bytes) {
        if (bytes)
            std::memcpy(blob.data() + o, src, bytes);
    };
    put(o_recs, recs.data(), recs.size() * sizeof(TensorRec));
    put(o_chunks, slots.data(), slots.size() * sizeof(ChunkRec));
    put(o_begin, chunk_begin.data(), chunk_begin.size() * sizeof(int32_t));
    put(o_segs, segs.data(), segs.size() * sizeof(int2));
    put(o_segbegin, seg_begin.data(), seg_begin.size() * sizeof(int32_t));
    put(o_tcb, tensor_chunk_begin.data(), tensor_chunk_begin.size() * sizeof(int32_t));
    put(o_aggc, agg_chunks.data(), agg_chunks.size() * sizeof(AggChunkRec));
    put(o_aggf, fine_striped.data(), fine_striped.size() * sizeof(AggChunkRec));
    put(o_gac, ga_chunks.data(), ga_chunks.size() * sizeof(AggChunkRec));
    put(o_sbegin, sync_begin.data(), sync_begin.size() * sizeof(int32_t));
    put(o_ssegs, sync_segs.data(), sync_segs.size() * sizeof(int2));
    put(o_ssegbegin, sync_seg_begin.data(), sync_seg_begin.size() * sizeof(int32_t));
    put(o_stb, sync_tensor_begin.data(), sync_tensor_begin.size() * sizeof(int32_t));
    put(o_aw, agg_w.data(), agg_w.size() * sizeof(float *));
    put(o_ac, agg_c.data(), agg_c.size() * sizeof(uint16_t *));
    put(o_ag, agg_g.data(), agg_g.size() * sizeof(float *));
    put(o_agc, agg_gc.data(), agg_gc.size() * sizeof(uint16_t *));
    put(o_agrad, agg_grad.data(), agg_grad.size() * sizeof(void *));
    put(o_am, agg_m.data(), agg_m.size() * sizeof(float *));

    hipError_t e = hipMalloc(&plan->d_blob, off);
    if (e == hipSuccess)
        e = hipMemcpy(plan->d_blob, blob.data(), off, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        return fail(ctx, e == hipErrorOutOfMemory ? SELSYNC_ERR_OOM : SELSYNC_ERR_HIP, "plan tables: %s",
                    hipGetErrorString(e));
    }
    char *b = static_cast<char *>(plan->d_blob);
    plan->d_recs = reinterpret_cast<TensorRec *>(b + o_recs);
    plan->tab.recs = plan->d_recs;
    plan->tab.slots = reinterpret_cast<ChunkRec *>(b + o_chunks);
    plan->tab.partials = reinterpret_cast<double *>(b + o_part);
    plan->tab.nchunks = nchunks;
    plan->tab.nslots = nslots;
    plan->tab.per = per;
    plan->tab.chunk_elems = (uint32_t)chunk;
    plan->tab.has_momentum = momenta != nullptr;
    plan->d_chunk_begin = reinterpret_cast<int32_t *>(b + o_begin);
    plan->n_segs = (int)segs.size();
    plan->d_segs = reinterpret_cast<int2 *>(b + o_segs);
    plan->d_seg_sums = reinterpret_cast<double *>(b + o_segsum);
    plan->d_seg_begin = reinterpret_cast<int32_t *>(b + o_segbegin);
    plan->d_tensor_chunk_begin = reinterpret_cast<int32_t *>(b + o_tcb);
    plan->d_tensor_norms = reinterpret_cast<double *>(b + o_tnorm);
    // one-wave workgroups go with pieces of less than one coarse tile
    plan->t_agg.recs = reinterpret_cast<AggChunkRec *>(b + o_aggc);
    plan->t_agg.nslots = (int)agg_chunks.size();
    plan->t_agg.shape = agg_chunk < kAggTileElems ? kAggFine : kAggCoarse;
    plan->t_fine.recs = reinterpret_cast<AggChunkRec *>(b + o_aggf);
    plan->t_fine.nslots = np_pad;
    plan->t_fine.per8 = per8;
    plan->t_fine.shape = kAggFine;
    plan->t_ga.recs = reinterpret_cast<AggChunkRec *>(b + o_gac);
    plan->t_ga.nslots = (int)ga_chunks.size();
    plan->t_ga.shape = ga_chunk < kAggTileElems ? kAggFine : kAggCoarse;
    plan->d_sync_partials = reinterpret_cast<double *>(b + o_spart);
    plan->sync_per = K * per8;
    plan->d_sync_begin = reinterpret_cast<int32_t *>(b + o_sbegin);
    plan->n_sync_segs = (int)sync_segs.size();
    plan->d_sync_segs = reinterpret_cast<int2 *>(b + o_ssegs);
    plan->d_sync_seg_sums = reinterpret_cast<double *>(b + o_ssegsum);
    plan->d_sync_seg_begin = reinterpret_cast<int32_t *>(b + o_ssegbegin);
    plan->d_sync_tensor_begin = reinterpret_cast<int32_t *>(b + o_stb);
    plan->agg.w = reinterpret_cast<float *const *>(b + o_aw);
    plan->agg.lowp = reinterpret_cast<uint16_t *const *>(b + o_ac);
    plan->agg.global = reinterpret_cast<float *const *>(b + o_ag);
    plan->agg.glowp = reinterpret_cast<uint16_t *const *>(b + o_agc);
    plan->agg.g = reinterpret_cast<const void *const *>(b + o_agrad);
    plan->agg.m = reinterpret_cast<float *const *>(b + o_am);
    plan->d_agg_v = reinterpret_cast<float **>(b + o_av);
    plan->agg.v = plan->d_agg_v;

    ctx->live_plans += 1;
    *out = plan.release();
    return SELSYNC_OK;
}
}  // namespace

extern "C" int32_t selsync_plan_destroy(selsync_plan *plan)
{
    if (!plan)
        return SELSYNC_OK;
    (void)hipDeviceSynchronize();
    if (plan->ctx)
        plan->ctx->live_plans -= 1;
    delete plan;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_plan_info(const selsync_plan *plan, int32_t *num_tensors, int64_t *num_params,
                                     int32_t *update_chunks, int32_t *aggregate_chunks)
{
    if (!plan)
        return SELSYNC_ERR_INVALID_ARG;
    if (num_tensors)
        *num_tensors = plan->T;
    if (num_params)
        *num_params = plan->P;
    if (update_chunks)
        *update_chunks = plan->n_upd_chunks;
    if (aggregate_chunks)
        *aggregate_chunks = plan->n_agg_chunks;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_chunk_table_preview(const int64_t *numel, const int32_t *lead_elems, int32_t num_tensors,
                                               int32_t chunk_elems, int32_t capacity, int32_t *tensor_out,
                                               int64_t *offset_out, int32_t *count_out, int32_t *num_chunks)
{
    if (!num_chunks || num_tensors < 0 || (num_tensors > 0 && !numel))
        return SELSYNC_ERR_INVALID_ARG;
    const int chunk = chunk_elems > 0 ? chunk_elems : kDefaultChunkElems;
    if (chunk % kChunkGranule != 0 || chunk > (1 << 24))
        return SELSYNC_ERR_INVALID_ARG;
    int64_t total = 0;
    for (int t = 0; t < num_tensors; ++t) {
        if (numel[t] < 0)
            return SELSYNC_ERR_INVALID_ARG;
        const int lead = lead_elems ? lead_elems[t] : 0;
        if (lead < 0 || lead >= chunk)
            return SELSYNC_ERR_INVALID_ARG;
        split_tensor(numel[t], chunk, lead, [&](int64_t off, int64_t n, int64_t) {
            if (total < capacity) {
                if (tensor_out)
                    tensor_out[total] = t;
                if (offset_out)
                    offset_out[total] = off;
                if (count_out)
                    count_out[total] = (int32_t)n;
            }
            ++total;
        });
    }
    if (total > INT32_MAX)
        return SELSYNC_ERR_INVALID_ARG;
    *num_chunks = (int32_t)total;
    return SELSYNC_OK;
}

// =============================================================================== per-step path

extern "C" int32_t selsync_track_grad_change(selsync_ctx *ctx, selsync_plan *plan, float grad_scale, void *stream,
                                             int32_t blocking, double *norm_sq_out, double *delta_out,
                                             int32_t *flags_out, int32_t *sync_out)
{
    int32_t rc = check_plan(ctx, plan, true);
    if (rc)
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    SgdArgs a{0.f, 0.f, 0.f, grad_scale, 0};
    {
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_stream(kNormOnly, plan->mixed, plan->tab, a, plan->nontemporal, s));
    }
    if ((rc = enqueue_track(ctx, plan, s)))
        return rc;
    if (blocking)
        return fetch_decision(ctx, s, norm_sq_out, delta_out, flags_out, sync_out, nullptr);
    return SELSYNC_OK;
}

namespace {
// a4.  mode 0 follows the device-side decision: the launch is shaped for a cheap exit (few, large
// workgroups), because on most steps it only reads the decision.  When the launch is expected to
// work -- mode 1, or a last decision taken under a threshold of 0, where every step synchronises --
// it takes single-wavefront workgroups of 256 elements instead (73 % against 71 % of HBM peak).
int32_t enqueue_aggregate(selsync_ctx *ctx, selsync_plan *plan, int mode, hipStream_t s)
{
    ProfScope p(ctx, 2, s);
    // The kernel always gets the caller's mode: under mode 0 it follows the device-side decision word
    // whatever the host expects, so a launch recorded into a graph stays correct when the threshold
    // changes between replays.  The expectation only selects the table and workgroup shape.
    if (mode == 1 || expect_sync(ctx)) {
        HIP_TRY(ctx, launch_aggregate(plan->mixed, plan->t_fine, plan->agg, plan->K, &ctx->td.out->sync, mode,
                                      plan->nontemporal, s));
        return SELSYNC_OK;
    }
    HIP_TRY(ctx, launch_aggregate(plan->mixed, plan->t_agg, plan->agg, plan->K, &ctx->td.out->sync, mode,
                                  plan->nontemporal, s));
    return SELSYNC_OK;
}
}  // namespace

extern "C" int32_t selsync_local_step(selsync_ctx *ctx, selsync_plan *plan, const selsync_sgd *sgd, void *stream)
{
    int32_t rc = check_plan(ctx, plan, true);
    if (rc)
        return rc;
    SgdArgs a;
    if ((rc = resolve_sgd(ctx, plan, sgd, &a)))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    {
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_stream(kUpdateOnly, plan->mixed, plan->tab, a, plan->nontemporal, s));
    }
    ctx->local_steps += 1;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_aggregate_params(selsync_ctx *ctx, selsync_plan *plan, int32_t mode, void *stream)
{
    int32_t rc = check_plan(ctx, plan, false);
    if (rc)
        return rc;
    if (mode != 0 && mode != 1)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "mode must be 0 (if flagged) or 1 (always)");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((rc = enqueue_aggregate(ctx, plan, mode, s)))
        return rc;
    return SELSYNC_OK;
}

namespace {
// One pass: per-worker norm partials + local update + unconditional mean into every replica and the
// global model, then the tracker over that pass's partials.
int32_t enqueue_sync_step(selsync_ctx *ctx, selsync_plan *plan, const SgdArgs &a, hipStream_t s)
{
    {
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_sync_step(plan->mixed, plan->has_momenta, plan->t_fine, plan->agg, plan->K, a,
                                      plan->d_sync_partials, plan->nontemporal, s));
    }
    ctx->local_steps += 1;
    return enqueue_track(ctx, plan, s, true);
}

bool stream_is_capturing(hipStream_t s)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) {
        (void)hipGetLastError();
        return true;        // unknown: take the path that is right under any later threshold
    }
    return st != hipStreamCaptureStatusNone;
}
}  // namespace

extern "C" int32_t selsync_step_bsp(selsync_ctx *ctx, selsync_plan *plan, const selsync_sgd *sgd, void *stream,
                                    int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                                    int32_t *sync_out)
{
    int32_t rc = check_plan(ctx, plan, true);
    if (rc)
        return rc;
    SgdArgs a;
    if ((rc = resolve_sgd(ctx, plan, sgd, &a)))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((rc = enqueue_sync_step(ctx, plan, a, s)))
        return rc;
    if (blocking)
        return fetch_decision(ctx, s, norm_sq_out, delta_out, flags_out, sync_out, nullptr);
    return SELSYNC_OK;
}

extern "C" int32_t selsync_step(selsync_ctx *ctx, selsync_plan *plan, const selsync_sgd *sgd, void *stream,
                                int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                                int32_t *sync_out)
{
    int32_t rc = check_plan(ctx, plan, true);
    if (rc)
        return rc;
    SgdArgs a;
    if ((rc = resolve_sgd(ctx, plan, sgd, &a)))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Under a threshold of 0 every step synchronises (Delta >= 0 always holds): the one-pass kernel gives
    // the same tensors and decisions with 20K+4 instead of 28K+4 bytes per parameter.  Not while the
    // stream is being captured: a recorded launch must stay right if the threshold changes before a replay.
    if (ctx->cfg.delta == 0.0 && !stream_is_capturing(s)) {
        if ((rc = enqueue_sync_step(ctx, plan, a, s)))
            return rc;
        if (blocking)
            return fetch_decision(ctx, s, norm_sq_out, delta_out, flags_out, sync_out, nullptr);
        return SELSYNC_OK;
    }
    {
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_stream(kUpdateAndNorm, plan->mixed, plan->tab, a, plan->nontemporal, s));
    }
    ctx->local_steps += 1;
    if ((rc = enqueue_track(ctx, plan, s)))
        return rc;
    if ((rc = enqueue_aggregate(ctx, plan, 0, s)))
        return rc;
    if (blocking)
        return fetch_decision(ctx, s, norm_sq_out, delta_out, flags_out, sync_out, nullptr);
    return SELSYNC_OK;
}

// =============================================================================== data partitioning (Sec. III-D)

namespace {
int32_t partition_count(int64_t D, int32_t N, int32_t n, int32_t scheme, int64_t *count)
{
    if (D < 0 || N < 1 || n < 0 || n >= N || (scheme != 0 && scheme != 1) || !count)
        return SELSYNC_ERR_INVALID_ARG;
    *count = scheme == 1 ? D : chunk_start(D, N, (int64_t)n + 1) - chunk_start(D, N, n);
    return SELSYNC_OK;
}
}  // namespace

extern "C" int32_t selsync_partition_order(int64_t num_samples, int32_t num_workers, int32_t worker, int32_t scheme,
                                           int64_t capacity, int64_t *out, int64_t *count)
{
    if (!out && !count)
        return SELSYNC_ERR_INVALID_ARG;
    int64_t c = 0;
    int32_t rc = partition_count(num_samples, num_workers, worker, scheme, &c);
    if (rc)
        return rc;
    if (count)
        *count = c;
    if (out) {
        const int64_t lim = c < capacity ? c : capacity;
        for (int64_t p = 0; p < lim; ++p)
            out[p] = partition_index(num_samples, num_workers, worker, scheme, p);
    }
    return SELSYNC_OK;
}

extern "C" int32_t selsync_partition_order_device(int64_t num_samples, int32_t num_workers, int32_t worker,
                                                  int32_t scheme, int64_t capacity, int64_t *out_device,
                                                  int64_t *count, void *stream)
{
    int64_t c = 0;
    int32_t rc = partition_count(num_samples, num_workers, worker, scheme, &c);
    if (rc)
        return rc;
    if (count)
        *count = c;
    if (!out_device)
        return capacity > 0 && c > 0 ? SELSYNC_ERR_INVALID_ARG : SELSYNC_OK;
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, out_device) != hipSuccess || attr.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return SELSYNC_ERR_NOT_DEVICE_MEM;
    }
    const int64_t lim = c < capacity ? c : capacity;
    if (launch_partition_order(num_samples, num_workers, worker, scheme, lim, out_device,
                               static_cast<hipStream_t>(stream)) != hipSuccess)
        return SELSYNC_ERR_HIP;
    return SELSYNC_OK;
}

// =============================================================================== variant: Adam local update

namespace {
int32_t resolve_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *ad, AdamArgs *out)
{
    if (!ad)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "adam is NULL");
    if (!plan->has_second_moment)
        return fail(ctx, SELSYNC_ERR_STATE, "no second-moment buffers bound (selsync_plan_bind_second_moment)");
    if (!(ad->beta1 >= 0.0 && ad->beta1 < 1.0) || !(ad->beta2 >= 0.0 && ad->beta2 < 1.0))
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "betas must be in [0, 1)");
    const int64_t t = ad->step > 0 ? ad->step : ctx->local_steps + 1;
    out->lr = ad->lr;
    out->b1 = (float)ad->beta1;
    out->b2 = (float)ad->beta2;
    out->omb1 = (float)(1.0 - ad->beta1);
    out->omb2 = (float)(1.0 - ad->beta2);
    out->eps = ad->eps;
    out->wd = ad->weight_decay;
    out->gs = ad->grad_scale;
    out->bc1 = (float)(1.0 - std::pow(ad->beta1, (double)t));
    out->bc2 = (float)(1.0 - std::pow(ad->beta2, (double)t));
    out->first = t == 1 ? 1 : 0;
    return SELSYNC_OK;
}
}  // namespace

extern "C" int32_t selsync_plan_bind_second_moment(selsync_plan *plan, const selsync_tensor_list *v)
{
    return guarded(plan ? plan->ctx : nullptr, [&]() -> int32_t {
        if (!plan || !plan->ctx)
            return SELSYNC_ERR_INVALID_ARG;
        selsync_ctx *ctx = plan->ctx;
        int32_t rc = check_plan(ctx, plan, true, true);
        if (rc)
            return rc;
        if (!v)
            return fail(ctx, SELSYNC_ERR_INVALID_ARG, "second-moment lists are NULL");
        std::vector<Interval> ivals;
        if ((rc = check_lists(ctx, "second_moment", v, plan->K, plan->T, plan->numel, SELSYNC_F32, true, ivals)))
            return rc;
        for (int k = 0; k < plan->K; ++k)
            for (int t = 0; t < plan->T; ++t) {
                TensorRec &r = plan->h_recs[(size_t)k * plan->T + t];
                float *vp = static_cast<float *>(v[k].tensors[t].data);
                // if this tensor takes the vector path (all its streams share one address phase), the
                // second-moment buffer must share that phase too
                const int ph = stream_phase(r.w, 4);
                const bool vec = stream_phase(r.g, plan->mixed ? 2 : 4) == ph && stream_phase(r.m, 4) == ph &&
                                 (!plan->mixed || stream_phase(r.lowp, 2) == ph);
                if (plan->numel[t] > 0 && vec && stream_phase(vp, 4) != ph)
                    return fail(ctx, SELSYNC_ERR_INVALID_ARG,
                                "second_moment[%d] tensor %d must have the same address phase (mod 16 bytes) as its "
                                "momentum tensor", k, t);
            }
        // the new buffers are written: together with everything already bound they may not overlap
        std::vector<Interval> all = plan->ivals;
        all.insert(all.end(), ivals.begin(), ivals.end());
        if ((rc = check_overlap(ctx, all)))
            return rc;
        for (int k = 0; k < plan->K; ++k)
            for (int t = 0; t < plan->T; ++t)
                plan->h_recs[(size_t)k * plan->T + t].v = static_cast<float *>(v[k].tensors[t].data);
        (void)hipDeviceSynchronize();
        if (!plan->h_recs.empty()) {
            HIP_TRY(ctx, hipMemcpy(plan->d_recs, plan->h_recs.data(), plan->h_recs.size() * sizeof(TensorRec),
                                   hipMemcpyHostToDevice));
            std::vector<float *> vt((size_t)plan->T * plan->K);      // K-way kernels index t * K + k
            for (int k = 0; k < plan->K; ++k)
                for (int t = 0; t < plan->T; ++t)
                    vt[(size_t)t * plan->K + k] = static_cast<float *>(v[k].tensors[t].data);
            HIP_TRY(ctx, hipMemcpy(plan->d_agg_v, vt.data(), vt.size() * sizeof(float *), hipMemcpyHostToDevice));
        }
        plan->has_second_moment = true;      // plan->ivals stays the base set, so buffers can be re-bound
        return SELSYNC_OK;
    });
}

extern "C" int32_t selsync_local_step_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *adam,
                                           void *stream)
{
    int32_t rc = check_plan(ctx, plan, true, true);
    if (rc)
        return rc;
    AdamArgs a;
    if ((rc = resolve_adam(ctx, plan, adam, &a)))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    {
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_stream_adam(false, plan->mixed, plan->tab, a, plan->nontemporal, s));
    }
    ctx->local_steps += 1;
    return SELSYNC_OK;
}

namespace {
// One pass with Adam as the update: norm partials + Adam step of every worker + unconditional mean of the
// updated parameters (moment buffers stay per worker), then the tracker over that pass's partials.
int32_t enqueue_sync_step_adam(selsync_ctx *ctx, selsync_plan *plan, const AdamArgs &a, hipStream_t s)
{
    {
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_sync_step_adam(plan->mixed, plan->t_fine, plan->agg, plan->K, a, plan->d_sync_partials,
                                           plan->nontemporal, s));
    }
    ctx->local_steps += 1;
    return enqueue_track(ctx, plan, s, true);
}
}  // namespace

extern "C" int32_t selsync_step_bsp_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *adam, void *stream,
                                         int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                                         int32_t *sync_out)
{
    int32_t rc = check_plan(ctx, plan, true, true);
    if (rc)
        return rc;
    AdamArgs a;
    if ((rc = resolve_adam(ctx, plan, adam, &a)))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((rc = enqueue_sync_step_adam(ctx, plan, a, s)))
        return rc;
    if (blocking)
        return fetch_decision(ctx, s, norm_sq_out, delta_out, flags_out, sync_out, nullptr);
    return SELSYNC_OK;
}

extern "C" int32_t selsync_step_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *adam, void *stream,
                                     int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                                     int32_t *sync_out)
{
    int32_t rc = check_plan(ctx, plan, true, true);
    if (rc)
        return rc;
    AdamArgs a;
    if ((rc = resolve_adam(ctx, plan, adam, &a)))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (ctx->cfg.delta == 0.0 && !stream_is_capturing(s)) {      // every step synchronises: one pass (see selsync_step)
        if ((rc = enqueue_sync_step_adam(ctx, plan, a, s)))
            return rc;
        if (blocking)
            return fetch_decision(ctx, s, norm_sq_out, delta_out, flags_out, sync_out, nullptr);
        return SELSYNC_OK;
    }
    {
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_stream_adam(true, plan->mixed, plan->tab, a, plan->nontemporal, s));
    }
    ctx->local_steps += 1;
    if ((rc = enqueue_track(ctx, plan, s)))
        return rc;
    if ((rc = enqueue_aggregate(ctx, plan, 0, s)))
        return rc;
    if (blocking)
        return fetch_decision(ctx, s, norm_sq_out, delta_out, flags_out, sync_out, nullptr);
    return SELSYNC_OK;
}

// =============================================================================== variant: gradient aggregation

namespace {
// The update of a gradient-aggregation step.  Following the decision (mode 0) takes two
// predicated launches, of which exactly one does work: on "local" the streaming kernel in its
// fastest shape (each worker applies its own gradient), on "sync" the K-way kernel (every worker
// applies the mean gradient).  Mode 1 always aggregates.
int32_t enqueue_ga_update(selsync_ctx *ctx, selsync_plan *plan, const SgdArgs &a, int mode, hipStream_t s)
{
    if (mode == 1 || expect_sync(ctx)) {
        // One launch shaped for bandwidth.  Always-mode aggregates; otherwise (the last decision was taken
        // under a threshold of 0, so "sync" is expected) the kernel still reads the decision word and, should
        // it say "local", applies every worker's own gradient itself: right under any decision, also when a
        // recorded launch is replayed after the threshold has changed.
        ProfScope p(ctx, 2, s);
        HIP_TRY(ctx, launch_update_ga(plan->mixed, plan->has_momenta, plan->t_fine, plan->agg, plan->K,
                                      &ctx->td.out->sync, mode == 1 ? kGaAlways : kGaSyncOrLocal, a, plan->nontemporal, s));
        return SELSYNC_OK;
    }
    // Two launches that both follow the device-side decision word, of which exactly one works: on "local"
    // the streaming kernel in its fastest shape, on "sync" the K-way kernel.
    {
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_stream(kUpdateOnly, plan->mixed, plan->tab, a, plan->nontemporal, s, &ctx->td.out->sync, 0));
    }
    ProfScope p(ctx, 2, s);
    HIP_TRY(ctx, launch_update_ga(plan->mixed, plan->has_momenta, plan->t_ga, plan->agg, plan->K, &ctx->td.out->sync,
                                  kGaSyncOnly, a, plan->nontemporal, s));
    return SELSYNC_OK;
}

// The same structure with Adam as the update.
int32_t enqueue_ga_update_adam(selsync_ctx *ctx, selsync_plan *plan, const AdamArgs &a, int mode, hipStream_t s)
{
    if (mode == 1 || expect_sync(ctx)) {
        ProfScope p(ctx, 2, s);
        HIP_TRY(ctx, launch_update_ga_adam(plan->mixed, plan->t_fine, plan->agg, plan->K, &ctx->td.out->sync,
                                           mode == 1 ? kGaAlways : kGaSyncOrLocal, a, plan->nontemporal, s));
        return SELSYNC_OK;
    }
    {
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_stream_adam(false, plan->mixed, plan->tab, a, plan->nontemporal, s, &ctx->td.out->sync, 0));
    }
    ProfScope p(ctx, 2, s);
    HIP_TRY(ctx, launch_update_ga_adam(plan->mixed, plan->t_ga, plan->agg, plan->K, &ctx->td.out->sync, kGaSyncOnly, a,
                                       plan->nontemporal, s));
    return SELSYNC_OK;
}
}  // namespace

extern "C" int32_t selsync_ga_update(selsync_ctx *ctx, selsync_plan *plan, const selsync_sgd *sgd, int32_t mode,
                                     void *stream)
{
    int32_t rc = check_plan(ctx, plan, true);
    if (rc)
        return rc;
    if (mode != 0 && mode != 1)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "mode must be 0 (follow the decision) or 1 (always aggregate)");
    SgdArgs a;
    if ((rc = resolve_sgd(ctx, plan, sgd, &a)))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((rc = enqueue_ga_update(ctx, plan, a, mode, s)))
        return rc;
    ctx->local_steps += 1;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_step_ga(selsync_ctx *ctx, selsync_plan *plan, const selsync_sgd *sgd, void *stream,
                                   int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                                   int32_t *sync_out)
{
    int32_t rc = check_plan(ctx, plan, true);
    if (rc)
        return rc;
    SgdArgs a;
    if ((rc = resolve_sgd(ctx, plan, sgd, &a)))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    {
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_stream(kNormOnly, plan->mixed, plan->tab, a, plan->nontemporal, s));
    }
    if ((rc = enqueue_track(ctx, plan, s)))
        return rc;
    if ((rc = enqueue_ga_update(ctx, plan, a, 0, s)))
        return rc;
    ctx->local_steps += 1;
    if (blocking)
        return fetch_decision(ctx, s, norm_sq_out, delta_out, flags_out, sync_out, nullptr);
    return SELSYNC_OK;
}

extern "C" int32_t selsync_ga_update_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *adam, int32_t mode,
                                          void *stream)
{
    int32_t rc = check_plan(ctx, plan, true, true);
    if (rc)
        return rc;
    if (mode != 0 && mode != 1)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "mode must be 0 (follow the decision) or 1 (always aggregate)");
    AdamArgs a;
    if ((rc = resolve_adam(ctx, plan, adam, &a)))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((rc = enqueue_ga_update_adam(ctx, plan, a, mode, s)))
        return rc;
    ctx->local_steps += 1;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_step_ga_adam(selsync_ctx *ctx, selsync_plan *plan, const selsync_adam *adam, void *stream,
                                        int32_t blocking, double *norm_sq_out, double *delta_out, int32_t *flags_out,
                                        int32_t *sync_out)
{
    int32_t rc = check_plan(ctx, plan, true, true);
    if (rc)
        return rc;
    AdamArgs a;
    if ((rc = resolve_adam(ctx, plan, adam, &a)))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    {
        SgdArgs n{0.f, 0.f, 0.f, a.gs, 0, 0};      // the norm-only pass uses the gradient scale alone
        ProfScope p(ctx, 0, s);
        HIP_TRY(ctx, launch_stream(kNormOnly, plan->mixed, plan->tab, n, plan->nontemporal, s));
    }
    if ((rc = enqueue_track(ctx, plan, s)))
        return rc;
    if ((rc = enqueue_ga_update_adam(ctx, plan, a, 0, s)))
        return rc;
    ctx->local_steps += 1;
    if (blocking)
        return fetch_decision(ctx, s, norm_sq_out, delta_out, flags_out, sync_out, nullptr);
    return SELSYNC_OK;
}

// =============================================================================== observability

extern "C" int32_t selsync_read_decision(selsync_ctx *ctx, void *stream, double *norm_sq_out, double *delta_out,
                                         int32_t *flags_out, int32_t *sync_out)
{
    if (!ctx)
        return SELSYNC_ERR_INVALID_ARG;
    int32_t rc = check_device(ctx);
    if (rc)
        return rc;
    return fetch_decision(ctx, static_cast<hipStream_t>(stream), norm_sq_out, delta_out, flags_out, sync_out,
                          nullptr);
}

extern "C" int32_t selsync_read_tensor_norms(selsync_ctx *ctx, selsync_plan *plan, void *stream, double *out)
{
    int32_t rc = check_plan(ctx, plan, true);
    if (rc)
        return rc;
    if (!out)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "out is NULL");
    if (!plan->partials_valid)
        return fail(ctx, SELSYNC_ERR_STATE, "no tracking pass has run on this plan yet");
    const int n = plan->K * plan->T;
    if (n == 0)
        return SELSYNC_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan->partials_from_sync)
        HIP_TRY(ctx, launch_tensor_norms(plan->d_sync_partials, plan->sync_per, plan->d_sync_tensor_begin, n,
                                         plan->d_tensor_norms, s));
    else
        HIP_TRY(ctx, launch_tensor_norms(plan->tab.partials, plan->tab.per, plan->d_tensor_chunk_begin, n,
                                         plan->d_tensor_norms, s));
    HIP_TRY(ctx, hipMemcpyAsync(out, plan->d_tensor_norms, sizeof(double) * n, hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipStreamSynchronize(s));
    return SELSYNC_OK;
}

extern "C" int32_t selsync_get_stats(selsync_ctx *ctx, void *stream, selsync_stats *out)
{
    if (!ctx)
        return SELSYNC_ERR_INVALID_ARG;
    if (!out)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "out is NULL");
    int32_t rc = check_device(ctx);
    if (rc)
        return rc;
    DecisionHeader h;
    rc = fetch_decision(ctx, static_cast<hipStream_t>(stream), nullptr, nullptr, nullptr, nullptr, &h);
    if (rc != SELSYNC_OK && rc != SELSYNC_WARN_NONFINITE)
        return rc;
    out->steps_local = h.steps_local;
    out->steps_sync = h.steps_sync;
    const int64_t tot = h.steps_local + h.steps_sync;
    out->lssr = tot ? (double)h.steps_local / (double)tot : std::nan("");
    out->max_delta = h.max_delta;
    out->nonfinite_steps = h.nonfinite_steps;
    return SELSYNC_OK;
}

namespace {
struct StateHeader {
    uint64_t magic;
    int32_t num_workers, window;
    double alpha;
    int64_t local_steps;
    uint64_t payload_bytes;
    double delta;           // threshold in force (the device copy travels inside the payload)
    double tracked_delta;   // threshold under which the last decision was taken (-1: none)
    int32_t tracked;        // a decision exists
    int32_t reserved;
};
constexpr uint64_t kStateMagic = 0x53454c53594e4332ull;   // "SELSYNC2"
}  // namespace

extern "C" int32_t selsync_tracker_state_size(const selsync_ctx *ctx, int64_t *bytes)
{
    if (!ctx || !bytes)
        return SELSYNC_ERR_INVALID_ARG;
    *bytes = (int64_t)(sizeof(StateHeader) + ctx->state_bytes);
    return SELSYNC_OK;
}

extern "C" int32_t selsync_tracker_get_state(selsync_ctx *ctx, void *stream, void *buf, int64_t bytes)
{
    if (!ctx)
        return SELSYNC_ERR_INVALID_ARG;
    if (!buf || bytes < (int64_t)(sizeof(StateHeader) + ctx->state_bytes))
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "buffer is NULL or smaller than selsync_tracker_state_size");
    int32_t rc = check_device(ctx);
    if (rc)
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    StateHeader h{kStateMagic, ctx->cfg.num_workers, ctx->cfg.window, ctx->cfg.alpha, ctx->local_steps,
                  (uint64_t)ctx->state_bytes, ctx->cfg.delta, ctx->tracked_delta, ctx->tracked ? 1 : 0, 0};
    std::memcpy(buf, &h, sizeof h);
    HIP_TRY(ctx, hipMemcpyAsync(static_cast<char *>(buf) + sizeof h, ctx->d_state, ctx->state_bytes,
                                hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipStreamSynchronize(s));
    return SELSYNC_OK;
}

extern "C" int32_t selsync_tracker_set_state(selsync_ctx *ctx, void *stream, const void *buf, int64_t bytes)
{
    if (!ctx)
        return SELSYNC_ERR_INVALID_ARG;
    if (!buf || bytes < (int64_t)sizeof(StateHeader))
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "buffer is NULL or too small");
    StateHeader h;
    std::memcpy(&h, buf, sizeof h);
    if (h.magic != kStateMagic || h.num_workers != ctx->cfg.num_workers || h.window != ctx->cfg.window ||
        h.alpha != ctx->cfg.alpha || h.payload_bytes != ctx->state_bytes ||
        bytes < (int64_t)(sizeof h + h.payload_bytes) || !(h.delta >= 0.0))
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "state blob does not match this context (workers/window/alpha)");
    int32_t rc = check_device(ctx);
    if (rc)
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    HIP_TRY(ctx, hipMemcpyAsync(ctx->d_state, static_cast<const char *>(buf) + sizeof h, ctx->state_bytes,
                                hipMemcpyHostToDevice, s));
    HIP_TRY(ctx, hipStreamSynchronize(s));
    // the host's view follows the restored device state: threshold, whether a decision exists, and
    // the automatic first-step marker
    ctx->local_steps = h.local_steps;
    ctx->cfg.delta = h.delta;
    ctx->tracked = h.tracked != 0;
    ctx->tracked_delta = h.tracked_delta;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_profile_enable(selsync_ctx *ctx, int32_t enable, int32_t max_launches)
{
    return guarded(ctx, [&]() -> int32_t {
        if (!ctx)
            return SELSYNC_ERR_INVALID_ARG;
        int32_t rc = check_device(ctx);
        if (rc)
            return rc;
        if (!enable) {
            ctx->prof_on = false;
            return SELSYNC_OK;
        }
        if (max_launches < 1 || max_launches > (1 << 20))
            return fail(ctx, SELSYNC_ERR_INVALID_ARG, "max_launches out of range");
        for (int k = 0; k < 3; ++k) {
            while ((int)ctx->prof_pool[k].size() < max_launches) {
                ProfRec r;
                HIP_TRY(ctx, hipEventCreate(&r.start));
                hipError_t e = hipEventCreate(&r.stop);
                if (e != hipSuccess) {
                    (void)hipEventDestroy(r.start);
                    return fail(ctx, SELSYNC_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
                }
                ctx->prof_pool[k].push_back(r);
            }
            ctx->prof_used[k] = 0;
            ctx->prof_seen[k] = 0;
        }
        ctx->prof_cap = max_launches;
        ctx->prof_on = true;
        return SELSYNC_OK;
    });
}

extern "C" int32_t selsync_profile_config(selsync_ctx *ctx, int32_t kind_mask, int32_t stride)
{
    if (!ctx)
        return SELSYNC_ERR_INVALID_ARG;
    if (kind_mask < 0 || kind_mask > 7 || stride < 1)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "kind_mask must be in 0..7 and stride >= 1");
    ctx->prof_mask = kind_mask;
    ctx->prof_stride = stride;
    return SELSYNC_OK;
}

extern "C" int32_t selsync_profile_summary(selsync_ctx *ctx, int32_t kind, int64_t *count, double *total_ms)
{
    if (!ctx)
        return SELSYNC_ERR_INVALID_ARG;
    if (kind < 0 || kind > 2 || !count || !total_ms)
        return fail(ctx, SELSYNC_ERR_INVALID_ARG, "bad kind or NULL output");
    int32_t rc = check_device(ctx);
    if (rc)
        return rc;
    double tot = 0.0;
    const int n = ctx->prof_used[kind];
    for (int i = 0; i < n; ++i) {
        ProfRec &r = ctx->prof_pool[kind][i];
        HIP_TRY(ctx, hipEventSynchronize(r.stop));
        float ms = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&ms, r.start, r.stop));
        tot += ms;
    }
    *count = n;
    *total_ms = tot;
    ctx->prof_used[kind] = 0;
    return SELSYNC_OK;
}
