// Streaming ceilings of this GPU for the access mixes the LASGD kernels have:
// what rate does a kernel with no table look-ups, no tails and no arithmetic to
// speak of reach when it reads R arrays and writes W arrays of 800 MiB each?
// The library's kernels are judged against these figures as well as against the
// published 8 TB/s.  Every thread moves one 128-bit vector per array; the grid
// covers the arrays exactly (no persistent loop).
//
//   membench            prints one line per (pattern, workgroup size, streaming hint)
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                                  \
    do {                                                                                       \
        hipError_t e_ = (x);                                                                   \
        if (e_ != hipSuccess) {                                                                \
            printf("%s failed: %s\n", #x, hipGetErrorString(e_));                              \
            return 1;                                                                          \
        }                                                                                      \
    } while (0)

typedef float f4 __attribute__((ext_vector_type(4)));

template <bool NT> __device__ __forceinline__ f4 ld(const f4 *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT> __device__ __forceinline__ void st(f4 *p, f4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// R reads from a[0..R), W writes to a[R-W'..]: writes reuse the last W read arrays
// when INPLACE (the update pattern), else go to arrays of their own.
template <int R, int W, bool INPLACE, bool NT>
__global__ __launch_bounds__(256) void stream_kernel(f4 *base, size_t nvec, f4 *sink)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nvec) return;
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    f4 r[R > 0 ? R : 1];
#pragma unroll
    for (int k = 0; k < R; ++k) r[k] = ld<NT>(base + (size_t)k * nvec + i);
#pragma unroll
    for (int k = 0; k < R; ++k) acc += r[k];
    if constexpr (W == 0) {
        if (acc.x == 1.2345f) sink[threadIdx.x] = acc;       // never true: keeps the loads alive
    } else {
        const int first = INPLACE ? R - W : R;
#pragma unroll
        for (int k = 0; k < W; ++k) st<NT>(base + (size_t)(first + k) * nvec + i, acc * (0.5f + k));
    }
}

// ---- how the K replicas are spread over waves (the local-step mix, K = 8) ------------------
// Same bytes, same addresses; only the assignment of work to waves differs.
struct Rep { f4 *g, *x, *v; size_t stride, nvec; };          // replica k of an array at base + k*stride
__device__ __forceinline__ void update(f4 g, f4 &x, f4 &v)
{
    const f4 g1 = g + 1e-4f * x;
    v = 0.9f * v + g1;
    x = x - 0.1f * (g1 + 0.9f * v);
}
// one wave per (tile, replica): ORDER 0 = replica after replica, 1 = the replicas of a tile adjacent
template <int ORDER> __global__ __launch_bounds__(64) void rep_wave_kernel(Rep a)
{
    const size_t ntile = a.nvec / 64, item = blockIdx.x;
    const size_t k = ORDER == 0 ? item / ntile : item % 8, t = ORDER == 0 ? item % ntile : item / 8;
    const size_t o = k * a.stride + t * 64 + threadIdx.x;
    f4 g = ld<true>(a.g + o), x = ld<true>(a.x + o), v = ld<true>(a.v + o);
    update(g, x, v);
    st<true>(a.v + o, v);
    st<true>(a.x + o, x);
}
// one wave per tile walks the 8 replicas one after the other
__global__ __launch_bounds__(64) void rep_loop_kernel(Rep a)
{
    for (int k = 0; k < 8; ++k) {
        const size_t o = (size_t)k * a.stride + (size_t)blockIdx.x * 64 + threadIdx.x;
        f4 g = ld<true>(a.g + o), x = ld<true>(a.x + o), v = ld<true>(a.v + o);
        update(g, x, v);
        st<true>(a.v + o, v);
        st<true>(a.x + o, x);
    }
}
// one wave per tile issues all 24 loads, then all 16 stores
__global__ __launch_bounds__(64) void rep_all_kernel(Rep a)
{
    const size_t o = (size_t)blockIdx.x * 64 + threadIdx.x;
    f4 g[8], x[8], v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        g[k] = ld<true>(a.g + o + k * a.stride);
        x[k] = ld<true>(a.x + o + k * a.stride);
        v[k] = ld<true>(a.v + o + k * a.stride);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        update(g[k], x[k], v[k]);
        st<true>(a.v + o + k * a.stride, v[k]);
        st<true>(a.x + o + k * a.stride, x[k]);
    }
}

struct Case {
    const char *name;
    int reads, writes, arrays;
    void (*launch)(f4 *, size_t, f4 *, int, bool);
};

template <int R, int W, bool INPLACE>
void launch(f4 *base, size_t nvec, f4 *sink, int bs, bool nt)
{
    const dim3 grid((unsigned)((nvec + bs - 1) / bs)), block(bs);
    if (nt) hipLaunchKernelGGL((stream_kernel<R, W, INPLACE, true>), grid, block, 0, 0, base, nvec, sink);
    else hipLaunchKernelGGL((stream_kernel<R, W, INPLACE, false>), grid, block, 0, 0, base, nvec, sink);
}

int main()
{
    const size_t nvec = (size_t)50 * 1024 * 1024;                  // 800 MiB per array
    const size_t bytes = nvec * sizeof(f4);
    const Case cases[] = {
        {"read only (1R)", 1, 0, 1, launch<1, 0, false>},
        {"write only (1W)", 0, 1, 1, launch<0, 1, false>},
        {"copy (1R 1W)", 1, 1, 2, launch<1, 1, false>},
        {"local step (3R 2W in place)", 3, 2, 3, launch<3, 2, true>},
        {"step+merge (5R 3W in place)", 5, 3, 5, launch<5, 3, true>},
        {"mean, K=8 (8R 1W)", 8, 1, 9, launch<8, 1, false>},
    };
    f4 *buf = nullptr, *sink = nullptr;
    CK(hipMalloc(&buf, bytes * 9));
    CK(hipMalloc(&sink, 4096));
    CK(hipMemset(buf, 0, bytes * 9));
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    printf("device: %s, %d CUs; arrays of %zu MiB; one 128-bit vector per thread per array, grid = all vectors\n",
           prop.gcnArchName, prop.multiProcessorCount, bytes >> 20);
    printf("%-30s %5s %5s %10s %10s %10s\n", "pattern", "block", "hint", "best ms", "median ms", "GB/s(med)");
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    for (const Case &c : cases)
        for (int bs : {64, 128, 256})
            for (int nt = 0; nt < 2; ++nt) {
                float ms[15];
                for (int rep = -2; rep < 15; ++rep) {
                    CK(hipEventRecord(a));
                    c.launch(buf, nvec, sink, bs, nt != 0);
                    CK(hipGetLastError());
                    CK(hipEventRecord(b));
                    CK(hipEventSynchronize(b));
                    float t;
                    CK(hipEventElapsedTime(&t, a, b));
                    if (rep >= 0) ms[rep] = t;
                }
                for (int i = 0; i < 15; ++i)
                    for (int j = i + 1; j < 15; ++j)
                        if (ms[j] < ms[i]) { float t = ms[i]; ms[i] = ms[j]; ms[j] = t; }
                const double moved = (double)(c.reads + c.writes) * bytes;
                printf("%-30s %5d %5s %10.4f %10.4f %10.0f\n", c.name, bs, nt ? "nt" : "-", ms[0], ms[7], moved / ms[7] / 1e6);
            }
    // ---- K = 8 replicas of 100 MiB arrays g, x, v (24 x 100 MiB inside the same buffer) ----
    {
        const size_t rn = (size_t)25 * 1024 * 1024 / 4;                // vectors per replica-array
        Rep r{buf, buf + 8 * rn, buf + 16 * rn, rn, rn};
        const double moved = 5.0 * 8 * rn * sizeof(f4);
        const unsigned ntile = (unsigned)(rn / 64);
        printf("\nlocal-step mix over K = 8 replicas of 100 MiB arrays, 64-thread workgroups, hint nt: who does what\n");
        for (int variant = 0; variant < 4; ++variant) {
            float ms[11];
            for (int rep = -2; rep < 11; ++rep) {
                CK(hipEventRecord(a));
                if (variant == 0) hipLaunchKernelGGL(rep_wave_kernel<0>, dim3(ntile * 8), dim3(64), 0, 0, r);
                else if (variant == 1) hipLaunchKernelGGL(rep_wave_kernel<1>, dim3(ntile * 8), dim3(64), 0, 0, r);
                else if (variant == 2) hipLaunchKernelGGL(rep_loop_kernel, dim3(ntile), dim3(64), 0, 0, r);
                else hipLaunchKernelGGL(rep_all_kernel, dim3(ntile), dim3(64), 0, 0, r);
                CK(hipGetLastError());
                CK(hipEventRecord(b));
                CK(hipEventSynchronize(b));
                float t;
                CK(hipEventElapsedTime(&t, a, b));
                if (rep >= 0) ms[rep] = t;
            }
            for (int i = 0; i < 11; ++i)
                for (int j = i + 1; j < 11; ++j)
                    if (ms[j] < ms[i]) { float t = ms[i]; ms[i] = ms[j]; ms[j] = t; }
            const char *names[] = {"one wave per (tile, replica), replica after replica", "one wave per (tile, replica), replicas of a tile adjacent",
                                   "one wave per tile, loop over the replicas", "one wave per tile, all 24 loads then all 16 stores"};
            printf("%-60s %10.4f ms %8.0f GB/s\n", names[variant], ms[5], moved / ms[5] / 1e6);
        }
    }
    CK(hipFree(buf));
    CK(hipFree(sink));
    return 0;
}
