/*
 * LASGD CPU oracle -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, single-threaded restatement of what LASGD's per-iteration
 * update arithmetic computes, written from the paper:
 *   - local update        Algorithm 1 steps 3 and 7; optimizer per Sec. 5.2
 *   - "send to All-Reduce" Algorithm 1 steps 4 and 9c
 *   - the All-Reduce result  z_t = (1/P) sum_i x^i_t      (Sec. 3, Eq. 8)
 *   - global update       x^i_{t+1} = z_t + (x^i - x^i_t)  (Algorithm 1, 9a-b)
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may load
 * this file.  It shares no code with the HIP library.
 *
 * Precision.  The parameters are fp32 and the acceptance bar is stated per
 * fp32 parameter, so every function works on fp32 storage with ONE pinned
 * evaluation order (round-to-nearest-even, no flush-to-zero; fmaf() is the
 * correctly rounded fused multiply-add of C99).  The mean accumulates in
 * fp64 in replica order and rounds to fp32 once.  A second, independent
 * fp64 restatement lives in lasgd_ref64.py; the two are cross-checked.
 *
 * Pins (tests/test_oracle_pins.py): K=1 merge identity, zero-progress merge,
 * mean preservation, exact-rational brute force, the alpha=beta=1 special
 * case of Sec. 3 (Eq. 7-8), equivalence with torch.optim.SGD for identical
 * gradients, replica-mean trajectory = large-batch SGD, bf16 rounding vs
 * torch, mean vs exactly rounded sum.  Every function below is covered by at
 * least one of them; none is "parity unpinned".
 *
 * Extensions beyond the fixed-cadence algorithm (each pinned in
 * tests/test_oracle_ext_pins.py):
 *   - elastic coefficients alpha, beta of Sec. 3 (Eq. 5-6) in the asynchronous
 *     setting of Sec. 4
 *   - the mean over a subset of replicas (the partial All-Reduce of Sec. 6)
 *   - the SGD All-Reduce comparator of Sec. 2 / Table 1: one step on the mean gradient
 * Replica subsets and per-replica step counts / learning rates are handled by
 * the Python driver, which simply skips the replicas that are not taking part.
 *
 * Build: gcc -O2 -ffp-contract=off -fPIC -shared (contraction must stay off
 * so that only the fmaf() calls written here fuse).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ---- bf16 <-> fp32 ----------------------------------------------------- */

/* Round an fp32 value to bfloat16, nearest-even; NaN stays a (quiet) NaN. */
uint16_t lasgd_oracle_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)          /* NaN: keep sign, force quiet */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lower = u & 0xffffu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))
        upper += 1u;                               /* carries into exponent / inf correctly */
    return (uint16_t)upper;
}

/* bf16 -> fp32 is exact: the 16 bits become the high half of the fp32. */
float lasgd_oracle_bf16_widen(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* ---- local update (Algorithm 1 steps 3, 7; Sec. 5.2) ------------------- */
/*
 * The algorithm box writes plain SGD, x <- x - eta*g; the experiments use
 * Nesterov momentum and weight decay.  Taken in the usual framework
 * convention: L2 decay folded into the gradient, zero dampening, momentum
 * buffer starting at zero:
 *     g' = g + wd*x
 *     v  = mu*v + g'
 *     d  = g' + mu*v   (Nesterov)   or   d = v   (heavy ball)
 *     x  = x - eta*d
 * With mu = 0 and wd = 0 this is exactly step 7 of the box.
 */
static inline void step_one(float *x, float *v, float g, float lr, float mu,
                            float wd, int nesterov)
{
    float g1 = fmaf(wd, *x, g);
    float vn = fmaf(mu, *v, g1);
    float d = nesterov ? fmaf(mu, vn, g1) : vn;
    *x = fmaf(-lr, d, *x);
    *v = vn;
}

void lasgd_oracle_local_step_f32(float *x, float *v, const float *g, int64_t n,
                                 float lr, float mu, float wd, int nesterov)
{
    for (int64_t e = 0; e < n; ++e)
        step_one(&x[e], &v[e], g[e], lr, mu, wd, nesterov);
}

/* bf16 storage: x32 is the fp32 master the update acts on, g16 the bf16
 * gradient (widened exactly), x16 the bf16 copy of the new master. */
void lasgd_oracle_local_step_bf16(float *x32, uint16_t *x16, float *v,
                                  const uint16_t *g16, int64_t n, float lr,
                                  float mu, float wd, int nesterov)
{
    for (int64_t e = 0; e < n; ++e) {
        step_one(&x32[e], &v[e], lasgd_oracle_bf16_widen(g16[e]), lr, mu, wd, nesterov);
        x16[e] = lasgd_oracle_bf16_rne(x32[e]);
    }
}

/* ---- send to All-Reduce (Algorithm 1 steps 4, 9c) ---------------------- */
/* The model handed to the All-Reduce must be kept: step 9a subtracts it. */
void lasgd_oracle_snapshot(float *s, const float *x, int64_t n)
{
    for (int64_t e = 0; e < n; ++e)
        s[e] = x[e];
}

/* ---- the All-Reduce result (Sec. 3, Eq. 8) ----------------------------- */
/* z = (1/K) sum_k s[k], fp64 accumulation in replica order, one rounding. */
void lasgd_oracle_average(float *z, const float *const *s, int32_t K, int64_t n)
{
    for (int64_t e = 0; e < n; ++e) {
        double acc = 0.0;
        for (int32_t k = 0; k < K; ++k)
            acc += (double)s[k][e];
        z[e] = (float)(acc / (double)K);
    }
}

/* ---- global update (Algorithm 1 step 9a-b, optionally 9c) -------------- */
/* x <- z + (x - s), parenthesised as printed; then, if asked, s <- x. */
void lasgd_oracle_merge_f32(float *x, float *s, const float *z, int64_t n,
                            int resnapshot)
{
    for (int64_t e = 0; e < n; ++e) {
        float progress = x[e] - s[e];
        float xn = z[e] + progress;
        x[e] = xn;
        if (resnapshot)
            s[e] = xn;
    }
}

void lasgd_oracle_merge_bf16(float *x32, uint16_t *x16, float *s, const float *z,
                             int64_t n, int resnapshot)
{
    for (int64_t e = 0; e < n; ++e) {
        float progress = x32[e] - s[e];
        float xn = z[e] + progress;
        x32[e] = xn;
        x16[e] = lasgd_oracle_bf16_rne(xn);
        if (resnapshot)
            s[e] = xn;
    }
}

/* bf16 storage start-up: the master is the exact widening of the params. */
void lasgd_oracle_widen_bf16(float *x32, const uint16_t *x16, int64_t n)
{
    for (int64_t e = 0; e < n; ++e)
        x32[e] = lasgd_oracle_bf16_widen(x16[e]);
}

/* ---- elastic averaging with general alpha, beta (Sec. 3, Eq. 5-6) ------- */
/*
 * Centre update, Eq. 5 read with beta_t = P*gamma_t:  z <- (1-beta)*z + beta*mean_k s[k].
 * The mean is taken over the models sent for this global update (the indexing
 * of Eq. 8 and Algorithm 1, not the one-step lag Eq. 5 prints).  fp64
 * throughout, one rounding to fp32.  beta = 1 is lasgd_oracle_average.
 */
void lasgd_oracle_average_elastic(float *z, const float *const *s, int32_t K, int64_t n, float beta)
{
    const double b = (double)beta, one_minus_b = 1.0 - (double)beta;
    for (int64_t e = 0; e < n; ++e) {
        double acc = 0.0;
        for (int32_t k = 0; k < K; ++k)
            acc += (double)s[k][e];
        double mean = acc / (double)K;
        double keep = one_minus_b * (double)z[e];
        double pull = b * mean;
        z[e] = (float)(keep + pull);
    }
}

/*
 * Local side, Eq. 6 carried to the asynchronous setting: the elastic pull
 * alpha*(z_t - x^i_t) is measured at the model that was sent and applied to the
 * model as it is now:  x <- x + alpha*(z - s).  With one step in flight
 * (x = s - eta*g) this is Eq. 6, alpha*z + (1-alpha)*s - eta*g; with alpha = 1
 * it is step 9a of Algorithm 1 up to rounding order (lasgd_oracle_merge_f32
 * keeps the printed parenthesisation for that case).
 */
void lasgd_oracle_merge_elastic_f32(float *x, float *s, const float *z, int64_t n, float alpha,
                                    int resnapshot)
{
    for (int64_t e = 0; e < n; ++e) {
        float pull = z[e] - s[e];
        float xn = fmaf(alpha, pull, x[e]);
        x[e] = xn;
        if (resnapshot)
            s[e] = xn;
    }
}

void lasgd_oracle_merge_elastic_bf16(float *x32, uint16_t *x16, float *s, const float *z, int64_t n,
                                     float alpha, int resnapshot)
{
    for (int64_t e = 0; e < n; ++e) {
        float pull = z[e] - s[e];
        float xn = fmaf(alpha, pull, x32[e]);
        x32[e] = xn;
        x16[e] = lasgd_oracle_bf16_rne(xn);
        if (resnapshot)
            s[e] = xn;
    }
}

/* ---- SGD All-Reduce comparator (Sec. 2; "SGD-AR" of Table 1) ------------ */
/*
 * All workers average their mini-batch gradients and every worker applies the
 * same step: gbar = (1/K) sum_k g[k] (fp64 in replica order, one rounding to
 * fp32), then the local update of Sec. 5.2 with gbar on each replica.
 */
void lasgd_oracle_mean_gradient_f32(float *gbar, const float *const *g, int32_t K, int64_t n)
{
    for (int64_t e = 0; e < n; ++e) {
        double acc = 0.0;
        for (int32_t k = 0; k < K; ++k)
            acc += (double)g[k][e];
        gbar[e] = (float)(acc / (double)K);
    }
}

void lasgd_oracle_mean_gradient_bf16(float *gbar, const uint16_t *const *g16, int32_t K, int64_t n)
{
    for (int64_t e = 0; e < n; ++e) {
        double acc = 0.0;
        for (int32_t k = 0; k < K; ++k)
            acc += (double)lasgd_oracle_bf16_widen(g16[k][e]);
        gbar[e] = (float)(acc / (double)K);
    }
}

/* the bf16-storage local step fed an fp32 gradient (the mean above) */
void lasgd_oracle_local_step_bf16_g32(float *x32, uint16_t *x16, float *v, const float *g, int64_t n,
                                      float lr, float mu, float wd, int nesterov)
{
    for (int64_t e = 0; e < n; ++e) {
        step_one(&x32[e], &v[e], g[e], lr, mu, wd, nesterov);
        x16[e] = lasgd_oracle_bf16_rne(x32[e]);
    }
}
