/*
 * A plain C consumer of the LASGD C ABI: no Python, no torch.  It allocates the
 * replicas' buffers with the HIP runtime, walks Algorithm 1 (prologue + T
 * iterations, global update every m) through include/lasgd.h, and compares
 * the state after every step with the CPU oracle (test infrastructure, linked
 * as a separate shared library), bit for bit.
 *
 * Usage: abi_check [K] [m] [T] [fused]      exit status 0 = all steps identical.
 * fused = 1: the global update and the next All-Reduce go out as one call,
 * lasgd_step_merge_average.  At the end the context-free, allocation-free
 * lasgd_global_update_static is checked on copies of the final state.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/lasgd.h"

/* the oracle's C entry points (oracle/lasgd_oracle.c) */
void lasgd_oracle_local_step_f32(float *x, float *v, const float *g, int64_t n, float lr, float mu, float wd, int nesterov);
void lasgd_oracle_snapshot(float *s, const float *x, int64_t n);
void lasgd_oracle_average(float *z, const float *const *s, int32_t K, int64_t n);
void lasgd_oracle_merge_f32(float *x, float *s, const float *z, int64_t n, int resnapshot);

#define HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); return 2; } } while (0)
#define LASGD(call) do { lasgd_status s_ = (call); if (s_ != LASGD_OK) { fprintf(stderr, "%s -> %d: %s\n", #call, (int)s_, lasgd_last_error(ctx)); return 3; } } while (0)

/* counter-based inputs: SplitMix64 of (seed, step, replica, element) mapped to a centred uniform */
static float draw(uint64_t seed, uint64_t step, uint64_t k, uint64_t e, float scale)
{
    uint64_t z = seed * 0x9E3779B97F4A7C15ull + step * 0xBF58476D1CE4E5B9ull + k * 0x94D049BB133111EBull + e;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return scale * ((float)(z >> 40) / 8388608.0f - 1.0f);
}

enum { NT = 4 };
static const int64_t numel[NT] = {5000, 3, 1024, 257};
static const float wd[NT] = {1e-4f, 0.0f, 1e-3f, 0.0f};

int main(int argc, char **argv)
{
    const int K = argc > 1 ? atoi(argv[1]) : 3, m = argc > 2 ? atoi(argv[2]) : 2, T = argc > 3 ? atoi(argv[3]) : 6;
    const int fused = argc > 4 ? atoi(argv[4]) : 0;
    const float lr = 0.05f, mu = 0.9f;
    int64_t N = 0, off[NT + 1];
    for (int t = 0; t < NT; ++t) { off[t] = N; N += numel[t]; }
    off[NT] = N;
    if (K < 1 || K > 64 || m < 1 || T < 0) { fprintf(stderr, "bad arguments\n"); return 1; }

    /* host state of the oracle */
    float **ox = calloc(K, sizeof *ox), **ov = calloc(K, sizeof *ov), **os = calloc(K, sizeof *os), **og = calloc(K, sizeof *og);
    float *oz = calloc(N, sizeof *oz), *tmp = calloc(N, sizeof *tmp);
    for (int k = 0; k < K; ++k) {
        ox[k] = calloc(N, sizeof(float)); ov[k] = calloc(N, sizeof(float));
        os[k] = calloc(N, sizeof(float)); og[k] = calloc(N, sizeof(float));
        for (int64_t e = 0; e < N; ++e) ox[k][e] = draw(1, 0, 0, e, 0.02f);       /* same model everywhere */
    }

    /* device buffers: one allocation per replica and kind, tensors on 256-byte boundaries */
    int64_t doff[NT + 1], dn = 0;
    for (int t = 0; t < NT; ++t) { doff[t] = dn; dn += (numel[t] + 63) / 64 * 64; }
    float **dx = calloc(K, sizeof *dx), **dg = calloc(K, sizeof *dg);
    hipStream_t main_s, side_s;
    HIP(hipStreamCreate(&main_s));
    HIP(hipStreamCreate(&side_s));
    lasgd_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.K = K; cfg.n_tensors = NT; cfg.numel = numel; cfg.storage = LASGD_F32;
    cfg.momentum = mu; cfg.nesterov = 1; cfg.weight_decay = wd;
    cfg.main_stream = main_s; cfg.side_stream = side_s;
    lasgd_ctx *ctx = NULL;
    lasgd_status st = lasgd_create(&cfg, &ctx);
    if (st != LASGD_OK) { fprintf(stderr, "lasgd_create -> %d: %s\n", (int)st, lasgd_last_error(NULL)); return 3; }
    for (int k = 0; k < K; ++k) {
        HIP(hipMalloc((void **)&dx[k], dn * sizeof(float)));
        HIP(hipMalloc((void **)&dg[k], dn * sizeof(float)));
        void *px[NT], *pg[NT];
        for (int t = 0; t < NT; ++t) {
            px[t] = dx[k] + doff[t]; pg[t] = dg[k] + doff[t];
            HIP(hipMemcpy(px[t], ox[k] + off[t], numel[t] * sizeof(float), hipMemcpyHostToDevice));
        }
        LASGD(lasgd_bind(ctx, k, px, pg));
    }

    int bad = 0, tau = 0;
    for (int step = 0; step <= T; ++step) {
        for (int k = 0; k < K; ++k) {
            for (int64_t e = 0; e < N; ++e) og[k][e] = draw(2, step, k, e, 1e-3f);
            for (int t = 0; t < NT; ++t)
                HIP(hipMemcpy(dg[k] + doff[t], og[k] + off[t], numel[t] * sizeof(float), hipMemcpyHostToDevice));
        }
        /* oracle */
        for (int k = 0; k < K; ++k)
            for (int t = 0; t < NT; ++t)
                lasgd_oracle_local_step_f32(ox[k] + off[t], ov[k] + off[t], og[k] + off[t], numel[t], lr, mu, wd[t], 1);
        int fire = 0;
        if (step == 0) { for (int k = 0; k < K; ++k) lasgd_oracle_snapshot(os[k], ox[k], N); fire = 1; }
        else if (++tau == m) { for (int k = 0; k < K; ++k) lasgd_oracle_merge_f32(ox[k], os[k], oz, N, 1); fire = 1; tau = 0; }
        if (fire) lasgd_oracle_average(oz, (const float *const *)os, K, N);
        /* library */
        if (step == 0) { LASGD(lasgd_local_step(ctx, lr)); LASGD(lasgd_snapshot(ctx)); LASGD(lasgd_average(ctx)); }
        else if (fire && fused) LASGD(lasgd_step_merge_average(ctx, lr));
        else if (fire) { LASGD(lasgd_step_merge(ctx, lr, 1)); LASGD(lasgd_average(ctx)); }
        else LASGD(lasgd_local_step(ctx, lr));
        /* compare */
        for (int which = LASGD_STATE_X; which <= LASGD_STATE_Z; ++which)
            for (int k = 0; k < (which == LASGD_STATE_Z ? 1 : K); ++k) {
                LASGD(lasgd_read_state(ctx, which, k, -1, tmp, N));
                const float *ref = which == LASGD_STATE_X ? ox[k] : which == LASGD_STATE_V ? ov[k] : which == LASGD_STATE_S ? os[k] : oz;
                for (int64_t e = 0; e < N; ++e)
                    if (memcmp(&tmp[e], &ref[e], 4) != 0 && !(tmp[e] == 0.0f && ref[e] == 0.0f)) {
                        if (bad < 5) fprintf(stderr, "step %d array %d replica %d element %lld: %.9g vs %.9g\n", step, which, k, (long long)e, tmp[e], ref[e]);
                        ++bad;
                    }
            }
    }
    int32_t done = 0;
    LASGD(lasgd_average_done(ctx, &done));

    /* the allocation-free global update on flat copies of the final models: pretend every replica made
     * one more bit of progress (x != s) and compare with the oracle's mean + global update */
    {
        float **fx = calloc(K, sizeof *fx), **fs = calloc(K, sizeof *fs);
        for (int k = 0; k < K; ++k) {
            for (int64_t e = 0; e < N; ++e) ox[k][e] += draw(3, 0, k, e, 1e-3f);
            HIP(hipMalloc((void **)&fx[k], N * sizeof(float)));
            HIP(hipMalloc((void **)&fs[k], N * sizeof(float)));
            HIP(hipMemcpy(fx[k], ox[k], N * sizeof(float), hipMemcpyHostToDevice));
            HIP(hipMemcpy(fs[k], os[k], N * sizeof(float), hipMemcpyHostToDevice));
        }
        lasgd_status gs = lasgd_global_update_static(K, N, fx, fs, 1, main_s);
        if (gs != LASGD_OK) { fprintf(stderr, "lasgd_global_update_static -> %d: %s\n", (int)gs, lasgd_last_error(NULL)); return 3; }
        HIP(hipStreamSynchronize(main_s));
        lasgd_oracle_average(oz, (const float *const *)os, K, N);
        for (int k = 0; k < K; ++k) lasgd_oracle_merge_f32(ox[k], os[k], oz, N, 1);
        for (int k = 0; k < K; ++k)
            for (int pass = 0; pass < 2; ++pass) {
                HIP(hipMemcpy(tmp, pass ? fs[k] : fx[k], N * sizeof(float), hipMemcpyDeviceToHost));
                const float *ref = pass ? os[k] : ox[k];
                for (int64_t e = 0; e < N; ++e)
                    if (memcmp(&tmp[e], &ref[e], 4) != 0 && !(tmp[e] == 0.0f && ref[e] == 0.0f)) {
                        if (bad < 5) fprintf(stderr, "static update, %s replica %d element %lld: %.9g vs %.9g\n", pass ? "sent" : "x", k, (long long)e, tmp[e], ref[e]);
                        ++bad;
                    }
            }
        for (int k = 0; k < K; ++k) { (void)hipFree(fx[k]); (void)hipFree(fs[k]); }
    }
    lasgd_destroy(ctx);
    for (int k = 0; k < K; ++k) { (void)hipFree(dx[k]); (void)hipFree(dg[k]); }
    printf("abi_check K=%d m=%d T=%d fused=%d N=%lld: %s (%d mismatching values)\n", K, m, T, fused, (long long)N, bad ? "FAIL" : "PASS", bad);
    return bad ? 4 : 0;
}
