/*
 * Sanitizer harness for the LASGD CPU oracle -- TEST INFRASTRUCTURE, not the product.
 *
 * Runs Algorithm 1 (Sec. 4) with a fixed cadence through the functions of
 * lasgd_oracle.c, then two steps of the SGD All-Reduce comparator (Sec. 2), on
 * inputs read from a file, and writes the final state to another file.  Built
 * by tests/test_oracle_sanitizers.py together with lasgd_oracle.c under
 * -fsanitize=address,undefined; every (replica, tensor, array) is a heap block
 * of exactly its size, so an access one element past any tensor is reported.
 * The test compares the output with the same schedule run through the regular
 * build of the oracle.
 *
 * Input file (little endian):
 *   int32  K, n_tensors, T, m, nesterov, bf16, elastic, reserved
 *   float  lr, mu, alpha, beta
 *   int64  numel[n_tensors]
 *   float  wd[n_tensors]
 *   x0:    per tensor, numel values (float, or uint16 bf16 patterns when bf16)
 *   grads: for step 0..T, for replica 0..K-1, per tensor, numel values (same type)
 * Output file: for k, for t: x; then v; then s; then z per tensor; then x16 (bf16 only);
 *   then x and v again after the two comparator steps (and x16 when bf16).
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

uint16_t lasgd_oracle_bf16_rne(float f);
float lasgd_oracle_bf16_widen(uint16_t h);
void lasgd_oracle_local_step_f32(float *x, float *v, const float *g, int64_t n, float lr, float mu, float wd, int nesterov);
void lasgd_oracle_local_step_bf16(float *x32, uint16_t *x16, float *v, const uint16_t *g16, int64_t n, float lr,
                                  float mu, float wd, int nesterov);
void lasgd_oracle_snapshot(float *s, const float *x, int64_t n);
void lasgd_oracle_average(float *z, const float *const *s, int32_t K, int64_t n);
void lasgd_oracle_merge_f32(float *x, float *s, const float *z, int64_t n, int resnapshot);
void lasgd_oracle_merge_bf16(float *x32, uint16_t *x16, float *s, const float *z, int64_t n, int resnapshot);
void lasgd_oracle_widen_bf16(float *x32, const uint16_t *x16, int64_t n);
void lasgd_oracle_average_elastic(float *z, const float *const *s, int32_t K, int64_t n, float beta);
void lasgd_oracle_merge_elastic_f32(float *x, float *s, const float *z, int64_t n, float alpha, int resnapshot);
void lasgd_oracle_merge_elastic_bf16(float *x32, uint16_t *x16, float *s, const float *z, int64_t n, float alpha,
                                     int resnapshot);
void lasgd_oracle_mean_gradient_f32(float *gbar, const float *const *g, int32_t K, int64_t n);
void lasgd_oracle_mean_gradient_bf16(float *gbar, const uint16_t *const *g16, int32_t K, int64_t n);
void lasgd_oracle_local_step_bf16_g32(float *x32, uint16_t *x16, float *v, const float *g, int64_t n, float lr,
                                      float mu, float wd, int nesterov);

static void die(const char *what)
{
    fprintf(stderr, "sanitize_driver: %s\n", what);
    exit(2);
}

static void *xmalloc(size_t n)
{
    void *p = malloc(n ? n : 1);
    if (!p) die("out of memory");
    return p;
}

static void rd(FILE *f, void *dst, size_t bytes)
{
    if (bytes && fread(dst, 1, bytes, f) != bytes) die("short input file");
}

static void wr(FILE *f, const void *src, size_t bytes)
{
    if (bytes && fwrite(src, 1, bytes, f) != bytes) die("short write");
}

int main(int argc, char **argv)
{
    if (argc != 3) die("usage: sanitize_driver <input> <output>");
    FILE *in = fopen(argv[1], "rb");
    if (!in) die("cannot open input");
    int32_t h[8];
    float p[4];
    rd(in, h, sizeof h);
    rd(in, p, sizeof p);
    const int32_t K = h[0], nt = h[1], T = h[2], m = h[3], nesterov = h[4], bf16 = h[5], elastic = h[6];
    const float lr = p[0], mu = p[1], alpha = p[2], beta = p[3];
    if (K < 1 || K > 64 || nt < 1 || nt > 4096 || T < 0 || m < 1) die("bad header");
    int64_t *numel = xmalloc(sizeof(int64_t) * nt);
    float *wd = xmalloc(sizeof(float) * nt);
    rd(in, numel, sizeof(int64_t) * nt);
    rd(in, wd, sizeof(float) * nt);
    const size_t gsz = bf16 ? 2 : 4;

    /* state: one exact-size block per (replica, tensor, array) */
    float **x = xmalloc(sizeof(float *) * K * nt), **v = xmalloc(sizeof(float *) * K * nt);
    float **s = xmalloc(sizeof(float *) * K * nt), **z = xmalloc(sizeof(float *) * nt);
    uint16_t **x16 = xmalloc(sizeof(uint16_t *) * K * nt);
    void **g = xmalloc(sizeof(void *) * K * nt);
    for (int t = 0; t < nt; ++t) {
        if (numel[t] < 1) die("bad numel");
        const size_t n = (size_t)numel[t];
        void *x0 = xmalloc(n * gsz);
        rd(in, x0, n * gsz);
        z[t] = xmalloc(n * 4);
        memset(z[t], 0, n * 4);
        for (int k = 0; k < K; ++k) {
            const int i = k * nt + t;
            x[i] = xmalloc(n * 4);
            v[i] = xmalloc(n * 4);
            s[i] = xmalloc(n * 4);
            x16[i] = xmalloc(n * 2);
            g[i] = xmalloc(n * gsz);
            memset(v[i], 0, n * 4);
            memset(s[i], 0, n * 4);
            if (bf16) {                                  /* step 1: same model everywhere */
                memcpy(x16[i], x0, n * 2);
                lasgd_oracle_widen_bf16(x[i], x16[i], (int64_t)n);
            } else {
                memcpy(x[i], x0, n * 4);
                memset(x16[i], 0, n * 2);
            }
        }
        free(x0);
    }
    int center_valid = 0, tau = 0;
    for (int step = 0; step <= T; ++step) {
        for (int k = 0; k < K; ++k)
            for (int t = 0; t < nt; ++t) rd(in, g[k * nt + t], (size_t)numel[t] * gsz);
        /* local update (steps 3 / 7) */
        for (int k = 0; k < K; ++k)
            for (int t = 0; t < nt; ++t) {
                const int i = k * nt + t;
                if (bf16) lasgd_oracle_local_step_bf16(x[i], x16[i], v[i], g[i], numel[t], lr, mu, wd[t], nesterov);
                else lasgd_oracle_local_step_f32(x[i], v[i], g[i], numel[t], lr, mu, wd[t], nesterov);
            }
        int fire = 0;
        if (step == 0) {
            for (int i = 0; i < K * nt; ++i) lasgd_oracle_snapshot(s[i], x[i], numel[i % nt]);   /* step 4 */
            fire = 1;
        } else if (++tau == m) {
            for (int k = 0; k < K; ++k)                                                           /* step 9a-c */
                for (int t = 0; t < nt; ++t) {
                    const int i = k * nt + t;
                    if (elastic && alpha != 1.0f) {
                        if (bf16) lasgd_oracle_merge_elastic_bf16(x[i], x16[i], s[i], z[t], numel[t], alpha, 1);
                        else lasgd_oracle_merge_elastic_f32(x[i], s[i], z[t], numel[t], alpha, 1);
                    } else {
                        if (bf16) lasgd_oracle_merge_bf16(x[i], x16[i], s[i], z[t], numel[t], 1);
                        else lasgd_oracle_merge_f32(x[i], s[i], z[t], numel[t], 1);
                    }
                }
            fire = 1;
            tau = 0;
        }
        if (fire) {                                                                               /* Eq. 8 */
            for (int t = 0; t < nt; ++t) {
                const float **sp = xmalloc(sizeof(float *) * K);
                for (int k = 0; k < K; ++k) sp[k] = s[k * nt + t];
                if (elastic && beta != 1.0f && center_valid) lasgd_oracle_average_elastic(z[t], sp, K, numel[t], beta);
                else lasgd_oracle_average(z[t], sp, K, numel[t]);
                free(sp);
            }
            center_valid = 1;
        }
    }
    FILE *out = fopen(argv[2], "wb");
    if (!out) die("cannot open output");
    for (int i = 0; i < K * nt; ++i) wr(out, x[i], (size_t)numel[i % nt] * 4);
    for (int i = 0; i < K * nt; ++i) wr(out, v[i], (size_t)numel[i % nt] * 4);
    for (int i = 0; i < K * nt; ++i) wr(out, s[i], (size_t)numel[i % nt] * 4);
    for (int t = 0; t < nt; ++t) wr(out, z[t], (size_t)numel[t] * 4);
    if (bf16)
        for (int i = 0; i < K * nt; ++i) wr(out, x16[i], (size_t)numel[i % nt] * 2);

    /* two comparator steps on the gradients still in g (the last step's) */
    for (int rep = 0; rep < 2; ++rep)
        for (int t = 0; t < nt; ++t) {
            float *gbar = xmalloc((size_t)numel[t] * 4);
            const void **gp = xmalloc(sizeof(void *) * K);
            for (int k = 0; k < K; ++k) gp[k] = g[k * nt + t];
            if (bf16) lasgd_oracle_mean_gradient_bf16(gbar, (const uint16_t *const *)gp, K, numel[t]);
            else lasgd_oracle_mean_gradient_f32(gbar, (const float *const *)gp, K, numel[t]);
            for (int k = 0; k < K; ++k) {
                const int i = k * nt + t;
                if (bf16) lasgd_oracle_local_step_bf16_g32(x[i], x16[i], v[i], gbar, numel[t], lr, mu, wd[t], nesterov);
                else lasgd_oracle_local_step_f32(x[i], v[i], gbar, numel[t], lr, mu, wd[t], nesterov);
            }
            free(gp);
            free(gbar);
        }
    for (int i = 0; i < K * nt; ++i) wr(out, x[i], (size_t)numel[i % nt] * 4);
    for (int i = 0; i < K * nt; ++i) wr(out, v[i], (size_t)numel[i % nt] * 4);
    if (bf16)
        for (int i = 0; i < K * nt; ++i) wr(out, x16[i], (size_t)numel[i % nt] * 2);
    /* the two scalar conversions, on a value that rounds up and one that is a tie */
    const uint16_t r1 = lasgd_oracle_bf16_rne(1.00390625f + 0.001f), r2 = lasgd_oracle_bf16_rne(1.00390625f);
    const float w1 = lasgd_oracle_bf16_widen(r1);
    wr(out, &r1, 2); wr(out, &r2, 2); wr(out, &w1, 4);
    fclose(out);
    fclose(in);
    for (int i = 0; i < K * nt; ++i) { free(x[i]); free(v[i]); free(s[i]); free(x16[i]); free(g[i]); }
    for (int t = 0; t < nt; ++t) free(z[t]);
    free(x); free(v); free(s); free(z); free(x16); free(g); free(numel); free(wd);
    return 0;
}
