/*
 * SelSync per-step hot path -- plain CPU oracle (TEST INFRASTRUCTURE, not product code).
 *
 * Slow, sequential, obviously-correct definitions of the four quantities the GPU
 * library computes each training step.  It shares no code with the HIP path and
 * must only be used by the tests, the smoke check and the CPU-baseline leg of the
 * benchmark.  Build: gcc -O2 -ffp-contract=off -fno-fast-math (no FMA contraction,
 * so every fp32 operation below rounds exactly once, in the order written).
 *
 *   a1  squared L2 norm of a gradient        Alg. 1 line 8 (the argument ||g_i||^2), Sec. III-A
 *   a2  smoothed relative gradient change     Eq. 2, EWMA paragraph of Sec. III-A, delta rule of Sec. III-B
 *   a3  local SGD update                      Alg. 1 line 9, optimiser recipes of Sec. IV-A
 *   a4  parameter aggregation                 Alg. 1 lines 14-15 and the mean formula in the Alg. 1 walkthrough
 *
 * Precision: norms, tracker and the replica mean accumulate in fp64; the update is
 * fp32 with one rounding per written operation.  Parity status: every function
 * here is pinned by tests/test_oracle_*.py against closed forms, exact rational
 * arithmetic, library routines (pandas ewm, torch.optim.SGD) and brute force.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ bf16 helpers */

/* bf16 -> fp32 is exact: the 16 stored bits are the high half of the fp32 pattern. */
float selsync_oracle_bf16_to_f32(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* fp32 -> bf16, round to nearest, ties to even; NaN stays a (quiet) NaN. */
uint16_t selsync_oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)          /* NaN: keep sign, force a quiet payload */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;                /* ties go to the even 16-bit pattern */
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* ------------------------------------------------------------------ a1: ||g||^2 */

/*
 * Continue a running squared-norm accumulation over one tensor.
 * acc_out = acc_in + sum_j (double)gh_j * (double)gh_j, j in index order, where
 * gh_j = fl32(grad_scale * g_j).  Calling it tensor after tensor with the running
 * value reproduces one flat index-order sum over the whole model (Alg. 1 line 8
 * passes the norm of the whole gradient).
 */
double selsync_oracle_norm_sq_accum_f32(double acc, const float *g, int64_t n, float grad_scale)
{
    for (int64_t j = 0; j < n; ++j) {
        float gh = grad_scale * g[j];
        acc += (double)gh * (double)gh;
    }
    return acc;
}

double selsync_oracle_norm_sq_accum_bf16(double acc, const uint16_t *g, int64_t n, float grad_scale)
{
    for (int64_t j = 0; j < n; ++j) {
        float gh = grad_scale * selsync_oracle_bf16_to_f32(g[j]);
        acc += (double)gh * (double)gh;
    }
    return acc;
}

/* ------------------------------------------------------------------ a3: local SGD update */

/*
 * Heavy-ball SGD with weight decay folded into the gradient (Alg. 1 line 9 with the
 * momentum / weight-decay recipes of Sec. IV-A), fp32, one rounding per operation:
 *     gh = fl(grad_scale * g)
 *     d  = fl(gh + fl(wd * w))
 *     m  = first ? d : fl(fl(mu * m) + d)
 *     w  = fl(w - fl(lr * m))
 */
void selsync_oracle_sgd_f32(float *w, float *m, const float *g, int64_t n,
                            float lr, float mu, float wd, float grad_scale, int first)
{
    for (int64_t j = 0; j < n; ++j) {
        float gh = grad_scale * g[j];
        float dec = wd * w[j];
        float d = gh + dec;
        float mom;
        if (first) {
            mom = d;
        } else {
            float mm = mu * m[j];
            mom = mm + d;
        }
        float stepv = lr * mom;
        m[j] = mom;
        w[j] = w[j] - stepv;
    }
}

/*
 * Mixed precision: bf16 gradient, fp32 master parameter and momentum, and a bf16
 * working copy of the parameter refreshed by round-to-nearest-even.
 */
void selsync_oracle_sgd_bf16(float *master, float *m, const uint16_t *g, uint16_t *copy, int64_t n,
                             float lr, float mu, float wd, float grad_scale, int first)
{
    for (int64_t j = 0; j < n; ++j) {
        float gh = grad_scale * selsync_oracle_bf16_to_f32(g[j]);
        float dec = wd * master[j];
        float d = gh + dec;
        float mom;
        if (first) {
            mom = d;
        } else {
            float mm = mu * m[j];
            mom = mm + d;
        }
        float stepv = lr * mom;
        m[j] = mom;
        master[j] = master[j] - stepv;
        copy[j] = selsync_oracle_f32_to_bf16(master[j]);
    }
}

/*
 * Momentum-free SGD (the Transformer recipe of Sec. IV-A names plain SGD with a decaying
 * learning rate and no momentum): no buffer at all,
 *     gh = fl(grad_scale * g);  d = fl(gh + fl(wd * w));  w = fl(w - fl(lr * d)).
 */
void selsync_oracle_sgd_plain_f32(float *w, const float *g, int64_t n, float lr, float wd, float grad_scale)
{
    for (int64_t j = 0; j < n; ++j) {
        float gh = grad_scale * g[j];
        float dec = wd * w[j];
        float d = gh + dec;
        float stepv = lr * d;
        w[j] = w[j] - stepv;
    }
}

void selsync_oracle_sgd_plain_bf16(float *master, const uint16_t *g, uint16_t *copy, int64_t n,
                                   float lr, float wd, float grad_scale)
{
    for (int64_t j = 0; j < n; ++j) {
        float gh = grad_scale * selsync_oracle_bf16_to_f32(g[j]);
        float dec = wd * master[j];
        float d = gh + dec;
        float stepv = lr * d;
        master[j] = master[j] - stepv;
        copy[j] = selsync_oracle_f32_to_bf16(master[j]);
    }
}

/*
 * Nesterov momentum (named among the optimisers in Sec. II-A; the paper gives no formula,
 * so this is the common look-ahead form): the buffer is updated as in plain momentum and
 * the step direction is the gradient plus mu times the NEW buffer,
 *     m = first ? d : fl(fl(mu * m) + d);  dir = fl(d + fl(mu * m));  w = fl(w - fl(lr * dir)).
 */
void selsync_oracle_sgd_nesterov_f32(float *w, float *m, const float *g, int64_t n,
                                     float lr, float mu, float wd, float grad_scale, int first)
{
    for (int64_t j = 0; j < n; ++j) {
        float gh = grad_scale * g[j];
        float dec = wd * w[j];
        float d = gh + dec;
        float mom;
        if (first) {
            mom = d;
        } else {
            float mm = mu * m[j];
            mom = mm + d;
        }
        float look = mu * mom;
        float dir = d + look;
        float stepv = lr * dir;
        m[j] = mom;
        w[j] = w[j] - stepv;
    }
}

void selsync_oracle_sgd_nesterov_bf16(float *master, float *m, const uint16_t *g, uint16_t *copy, int64_t n,
                                      float lr, float mu, float wd, float grad_scale, int first)
{
    for (int64_t j = 0; j < n; ++j) {
        float gh = grad_scale * selsync_oracle_bf16_to_f32(g[j]);
        float dec = wd * master[j];
        float d = gh + dec;
        float mom;
        if (first) {
            mom = d;
        } else {
            float mm = mu * m[j];
            mom = mm + d;
        }
        float look = mu * mom;
        float dir = d + look;
        float stepv = lr * dir;
        m[j] = mom;
        master[j] = master[j] - stepv;
        copy[j] = selsync_oracle_f32_to_bf16(master[j]);
    }
}

/* ------------------------------------------------------------------ a4: parameter aggregation */

/*
 * wbar_j = fl32( (sum_{k=0..K-1} (double)w_{k,j}) / K ), written to the global model
 * and to every replica (all workers pull the same averaged state).
 */
void selsync_oracle_average_f32(float *const *replicas, int K, float *global, int64_t n)
{
    for (int64_t j = 0; j < n; ++j) {
        double s = 0.0;
        for (int k = 0; k < K; ++k)
            s += (double)replicas[k][j];
        float mean = (float)(s / (double)K);
        global[j] = mean;
        for (int k = 0; k < K; ++k)
            replicas[k][j] = mean;
    }
}

/* Mixed precision: average the fp32 masters; refresh every bf16 copy from the mean. */
void selsync_oracle_average_bf16(float *const *masters, uint16_t *const *copies, int K,
                                 float *global_master, uint16_t *global_copy, int64_t n)
{
    for (int64_t j = 0; j < n; ++j) {
        double s = 0.0;
        for (int k = 0; k < K; ++k)
            s += (double)masters[k][j];
        float mean = (float)(s / (double)K);
        uint16_t h = selsync_oracle_f32_to_bf16(mean);
        global_master[j] = mean;
        global_copy[j] = h;
        for (int k = 0; k < K; ++k) {
            masters[k][j] = mean;
            copies[k][j] = h;
        }
    }
}

/* ------------------------------------------------------------------ variant: Adam local update */

/*
 * Adam (the optimiser of the AlexNet recipe in Sec. IV-A) as the local update of Alg. 1
 * line 9, fp32, one rounding per operation, in this order:
 *     gh = fl(grad_scale*g);  gd = fl(gh + fl(wd*w))
 *     m  = fl(fl(b1*m) + fl(omb1*gd));   v = fl(fl(b2*v) + fl(fl(omb2*gd)*gd))
 *     mh = fl(m/bc1);  vh = fl(v/bc2)
 *     w  = fl(w - fl(fl(lr*mh) / fl(sqrt(vh) + eps)))
 * omb1 = fl(1-b1), omb2 = fl(1-b2), bc1 = fl(1 - b1^t), bc2 = fl(1 - b2^t) are formed by the
 * caller (in double, rounded to fp32) for step t = 1, 2, ...; at t = 1 the buffers are taken
 * as zero whatever they hold.
 */
void selsync_oracle_adam_f32(float *w, float *m, float *v, const float *g, int64_t n, float lr, float b1, float b2,
                             float omb1, float omb2, float eps, float wd, float grad_scale, float bc1, float bc2,
                             int first)
{
    for (int64_t j = 0; j < n; ++j) {
        float gh = grad_scale * g[j];
        float dec = wd * w[j];
        float gd = gh + dec;
        float mo = first ? 0.0f : m[j];
        float vo = first ? 0.0f : v[j];
        float t1 = b1 * mo;
        float t2 = omb1 * gd;
        float mn = t1 + t2;
        float t3 = b2 * vo;
        float t4 = omb2 * gd;
        float t5 = t4 * gd;
        float vn = t3 + t5;
        float mh = mn / bc1;
        float vh = vn / bc2;
        float num = lr * mh;
        float den = sqrtf(vh) + eps;
        float q = num / den;
        m[j] = mn;
        v[j] = vn;
        w[j] = w[j] - q;
    }
}

void selsync_oracle_adam_bf16(float *master, float *m, float *v, const uint16_t *g, uint16_t *copy, int64_t n,
                              float lr, float b1, float b2, float omb1, float omb2, float eps, float wd,
                              float grad_scale, float bc1, float bc2, int first)
{
    for (int64_t j = 0; j < n; ++j) {
        float gh = grad_scale * selsync_oracle_bf16_to_f32(g[j]);
        float dec = wd * master[j];
        float gd = gh + dec;
        float mo = first ? 0.0f : m[j];
        float vo = first ? 0.0f : v[j];
        float t1 = b1 * mo;
        float t2 = omb1 * gd;
        float mn = t1 + t2;
        float t3 = b2 * vo;
        float t4 = omb2 * gd;
        float t5 = t4 * gd;
        float vn = t3 + t5;
        float mh = mn / bc1;
        float vh = vn / bc2;
        float num = lr * mh;
        float den = sqrtf(vh) + eps;
        float q = num / den;
        m[j] = mn;
        v[j] = vn;
        master[j] = master[j] - q;
        copy[j] = selsync_oracle_f32_to_bf16(master[j]);
    }
}

/* ------------------------------------------------------------------ variant: gradient aggregation */

/*
 * Gradient aggregation (Sec. III-C): on a synchronising step the workers exchange
 * gradients instead of parameters and every worker applies the same averaged gradient
 *     gbar_j = fl32( (sum_{k=0..K-1} (double)fl32(grad_scale * g_{k,j})) / K )
 * to its OWN parameters and momentum.  This only forms gbar; the update itself is
 * selsync_oracle_sgd_f32 (or its Nesterov form) with gbar as the gradient and grad_scale 1;
 * in mixed precision it acts on the fp32 masters and the bf16 copies are then refreshed
 * by rounding the masters.
 */
void selsync_oracle_average_grads_f32(const float *const *grads, int K, float grad_scale, float *gbar, int64_t n)
{
    for (int64_t j = 0; j < n; ++j) {
        double s = 0.0;
        for (int k = 0; k < K; ++k) {
            float gh = grad_scale * grads[k][j];
            s += (double)gh;
        }
        gbar[j] = (float)(s / (double)K);
    }
}

void selsync_oracle_average_grads_bf16(const uint16_t *const *grads, int K, float grad_scale, float *gbar, int64_t n)
{
    for (int64_t j = 0; j < n; ++j) {
        double s = 0.0;
        for (int k = 0; k < K; ++k) {
            float gh = grad_scale * selsync_oracle_bf16_to_f32(grads[k][j]);
            s += (double)gh;
        }
        gbar[j] = (float)(s / (double)K);
    }
}

/* ------------------------------------------------------------------ a2: significance tracker */

/*
 * One worker's RelativeGradChange state: the last <= window raw values of ||g||^2
 * (one is computed and kept per iteration: Alg. 1 line 8 and its walkthrough in
 * Sec. III-E) and the previous smoothed value.
 */
typedef struct selsync_oracle_tracker {
    int window;
    double alpha;
    double *hist;      /* hist[0] oldest ... hist[len-1] newest */
    int len;
    int has_prev;
    double s_prev;
} selsync_oracle_tracker;

selsync_oracle_tracker *selsync_oracle_tracker_new(int window, double alpha)
{
    if (window < 1)
        return NULL;
    selsync_oracle_tracker *t = (selsync_oracle_tracker *)calloc(1, sizeof *t);
    if (!t)
        return NULL;
    t->hist = (double *)calloc((size_t)window, sizeof(double));
    if (!t->hist) {
        free(t);
        return NULL;
    }
    t->window = window;
    t->alpha = alpha;
    return t;
}

void selsync_oracle_tracker_free(selsync_oracle_tracker *t)
{
    if (t) {
        free(t->hist);
        free(t);
    }
}

/*
 * Push this iteration's x = ||g_i||^2 and return Delta(g_i) (Eq. 2).
 *
 * Smoothed value: exponentially weighted moving average over the stored window,
 * newest sample weight 1, a sample of age j weight (1-alpha)^j, normalised by the
 * weight sum:   S_i = sum_j (1-alpha)^j x_{i-j} / sum_j (1-alpha)^j ,  j < min(i+1, window).
 * Relative change: |S_i - S_{i-1}| / S_{i-1}.
 * Conventions where the paper is silent: no previous value -> 0; 0/0 -> 0; a result
 * that is not a number (non-finite history) -> +infinity so the worker asks to sync.
 */
double selsync_oracle_tracker_push(selsync_oracle_tracker *t, double x, double *s_out)
{
    if (t->len == t->window) {
        memmove(t->hist, t->hist + 1, (size_t)(t->window - 1) * sizeof(double));
        t->len -= 1;
    }
    t->hist[t->len++] = x;

    double num = 0.0, den = 0.0;
    for (int j = 0; j < t->len; ++j) {
        double wgt = pow(1.0 - t->alpha, (double)j);
        num += wgt * t->hist[t->len - 1 - j];
        den += wgt;
    }
    double s = num / den;

    double delta;
    if (!t->has_prev) {
        delta = 0.0;
    } else if (t->s_prev == 0.0 && s == 0.0) {
        delta = 0.0;
    } else {
        delta = fabs(s - t->s_prev) / t->s_prev;
        if (isnan(delta))
            delta = INFINITY;
    }
    if (!isfinite(x))
        delta = INFINITY;

    t->s_prev = s;
    t->has_prev = 1;
    if (s_out)
        *s_out = s;
    return delta;
}

/* The delta rule: a worker raises its flag when Delta >= delta (Alg. 1 lines 10-11). */
int selsync_oracle_flag(double delta_g, double threshold)
{
    return delta_g >= threshold ? 1 : 0;
}
