// Device code of the LASGD update library (gfx950 / CDNA4, wave64).
//
// Everything here is bandwidth-bound streaming: a handful of fp32 FMAs per
// 20-28 bytes moved, so there is no matrix-core work.  What matters is that
// every lane moves 128 bits per access, that a wave covers a contiguous
// kilobyte per instruction, that many independent loads are in flight before
// the first use, and that the mean z (shared by all K replicas) is fetched
// once per tile and kept in registers while the wave walks the replicas.
//
// Arithmetic is pinned: contraction is off for this file, so only the
// __builtin_fmaf calls below fuse.  Local update: Algorithm 1 steps 3 and 7
// with the optimizer of Sec. 5.2; global update: step 9a-b; mean: Sec. 3 Eq. 8.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lasgd {

// One tile = up to 256*VEC consecutive elements of ONE tensor, handled by one
// wave: lane l owns elements [4l, 4l+4) of each 256-element row of the tile.
struct Tile {
    uint64_t toff;     // first element, relative to the tensor's start
    uint64_t aoff;     // first element, relative to a replica's start in the library arenas
    uint32_t tensor;   // index into the pointer tables
    uint32_t count;    // elements in this tile (<= 256*VEC; smaller only at a tensor's end)
    float wd;          // the tensor's weight decay
    uint32_t pad_;
};
static_assert(sizeof(Tile) == 32, "tile descriptors are two 16-byte loads");

// The descriptor and pointer tables are read with wave-uniform indices.  The
// compiler fetches them through the vector memory path (all lanes, one
// address).  Forcing scalar loads instead (constant address space) was
// measured 4.5 % slower on MI355X: every descriptor is used once, so each
// scalar load misses the small scalar cache, while the vector L1 keeps more
// of these misses in flight.
__device__ __forceinline__ Tile load_tile(const Tile *p) { return *p; }
__device__ __forceinline__ char *load_ptr(void *const *table, size_t i) { return static_cast<char *>(table[i]); }

enum Op : int { OP_STEP = 0, OP_MERGE = 1, OP_STEP_MERGE = 2, OP_SNAPSHOT = 3, OP_INIT = 4 };

struct ApplyArgs {
    const Tile *tiles;
    void *const *xptr;      // [K * n_tensors] caller's parameters (fp32 or bf16)
    void *const *gptr;      // [K * n_tensors] caller's gradients  (fp32 or bf16)
    float *x32;             // bf16 storage only: fp32 master, [K][npad]
    float *v;               // momentum,     [K][npad]
    float *s;               // sent models,  [K][npad]
    float *z;               // mean,         [npad] (written only by the fused step+update+mean kernel)
    uint64_t npad;          // elements per replica in the arenas
    uint32_t ntiles, K, n_tensors;
    uint32_t kper;          // replicas a wave handles back to back
    uint32_t kgroups;       // ceil(K / kper)
    uint32_t nitems;        // ntiles * kgroups
    float neg_lr, mu;
    int32_t nesterov, resnap;
    uint32_t chunk;         // item order, see apply_kernel
    uint32_t full_items;    // (ntiles / chunk) * chunk * kgroups
    uint32_t tail_first;    // first tile of the last, shorter chunk
    uint32_t tail_chunk;    // its length (>= 1 even when unused)
    uint32_t tail_stride;   // items per replica group in the last chunk: tail_chunk rounded up so that every
                            // group's pass starts on the same XCD; the items in between do nothing
    // the replica-group kernels finish a mean over all K replicas themselves
    int32_t use_mul;        // K is a power of two: multiply by the exact reciprocal
    double inv_k, k_as_double;
};

// What the extended entry points add: replicas that sit a call out, a step size
// per replica (eta is indexed by each node's own clock, Algorithm 1) and the
// elastic coefficient alpha of Sec. 3, Eq. 6.
struct ExtArgs {
    uint64_t step_mask;     // bit k: replica k takes the local update (or is snapshotted / initialised)
    uint64_t merge_mask;    // bit k: replica k takes the global update
    float alpha;            // 1 = step 9a of Algorithm 1 exactly
    float neg_lr_k[64];     // -eta per replica
};

// ---- 128-bit / 64-bit accesses, optionally with the streaming hint --------
// Every pointer the kernels dereference is device (global) memory.  Pointers
// that come out of the tables are generic as far as the compiler can tell and
// would be accessed with FLAT instructions; casting to the global address
// space makes every access a GLOBAL load or store.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
#define LASGD_GLOBAL_AS __attribute__((address_space(1)))
template <class T> __device__ __forceinline__ const LASGD_GLOBAL_AS T *as_global(const void *p)
{
    return reinterpret_cast<const LASGD_GLOBAL_AS T *>(reinterpret_cast<uintptr_t>(p));
}
template <class T> __device__ __forceinline__ LASGD_GLOBAL_AS T *as_global(void *p)
{
    return reinterpret_cast<LASGD_GLOBAL_AS T *>(reinterpret_cast<uintptr_t>(p));
}

template <int NT> __device__ __forceinline__ float4 ld4(const float *p)
{
    f32x4_t r;
    if constexpr (NT & 1) r = __builtin_nontemporal_load(as_global<f32x4_t>(p));
    else r = *as_global<f32x4_t>(p);
    return make_float4(r.x, r.y, r.z, r.w);
}
template <int NT> __device__ __forceinline__ void st4(float *p, float4 a)
{
    f32x4_t r = {a.x, a.y, a.z, a.w};
    if constexpr (NT & 2) __builtin_nontemporal_store(r, as_global<f32x4_t>(p));
    else *as_global<f32x4_t>(p) = r;
}
template <int NT> __device__ __forceinline__ uint2 ld2(const uint16_t *p)
{
    u32x2_t r;
    if constexpr (NT & 1) r = __builtin_nontemporal_load(as_global<u32x2_t>(p));
    else r = *as_global<u32x2_t>(p);
    return make_uint2(r.x, r.y);
}
template <int NT> __device__ __forceinline__ void st2(uint16_t *p, uint2 a)
{
    u32x2_t r = {a.x, a.y};
    if constexpr (NT & 2) __builtin_nontemporal_store(r, as_global<u32x2_t>(p));
    else *as_global<u32x2_t>(p) = r;
}

// ---- bf16 <-> fp32 ----------------------------------------------------------
__device__ __forceinline__ float bf16_widen(uint32_t h) { return __uint_as_float(h << 16); }

// Round to nearest, ties to even, by adding 0x7fff plus the kept LSB and
// truncating; NaN is kept a quiet NaN.
__device__ __forceinline__ uint32_t bf16_round(float f)
{
    uint32_t u = __float_as_uint(f);
    uint32_t r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    uint32_t nan = (u >> 16) | 0x40u;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? nan : r;
}
__device__ __forceinline__ float4 widen4(uint2 p)
{
    return make_float4(bf16_widen(p.x & 0xffffu), bf16_widen(p.x >> 16),
                       bf16_widen(p.y & 0xffffu), bf16_widen(p.y >> 16));
}
__device__ __forceinline__ uint2 round4(float4 a)
{
    return make_uint2(bf16_round(a.x) | (bf16_round(a.y) << 16),
                      bf16_round(a.z) | (bf16_round(a.w) << 16));
}

// ---- the arithmetic, one element -------------------------------------------
// Local update (Algorithm 1 step 7; Sec. 5.2): four fused multiply-adds.
__device__ __forceinline__ void step_elem(float &x, float &v, float g, float wd, float mu,
                                          float neg_lr, int nesterov)
{
    float g1 = __builtin_fmaf(wd, x, g);
    float vn = __builtin_fmaf(mu, v, g1);
    float d = nesterov ? __builtin_fmaf(mu, vn, g1) : vn;
    x = __builtin_fmaf(neg_lr, d, x);
    v = vn;
}
// Global update (step 9a): z + (x - s), parenthesised as printed.
__device__ __forceinline__ float merge_elem(float x, float s, float z)
{
    float progress = x - s;
    return z + progress;
}

// Elastic form (Eq. 6 in the asynchronous setting): the pull alpha*(z - s) is
// measured at the sent model and applied to the current one.  alpha == 1 keeps
// the printed form of step 9a, so both entry-point families agree bit for bit there.
__device__ __forceinline__ float merge_elem_elastic(float x, float s, float z, float alpha)
{
    float pulled = __builtin_fmaf(alpha, z - s, x);
    return alpha == 1.0f ? merge_elem(x, s, z) : pulled;
}

#define LASGD_FOR4(body)                                                                       \
    {                                                                                          \
        { constexpr int c = 0; body }                                                          \
        { constexpr int c = 1; body }                                                          \
        { constexpr int c = 2; body }                                                          \
        { constexpr int c = 3; body }                                                          \
    }
__device__ __forceinline__ float &comp(float4 &a, int c)
{
    return c == 0 ? a.x : c == 1 ? a.y : c == 2 ? a.z : a.w;
}
__device__ __forceinline__ float compv(const float4 &a, int c)
{
    return c == 0 ? a.x : c == 1 ? a.y : c == 2 ? a.z : a.w;
}

// Apply one operation to VEC rows of one replica's tile.  `rows` is the number
// of full 256-element rows (VEC on the fast path); `count` bounds the ragged
// path.  x/g point at the tile's first element in the caller's buffers
// (storage dtype), xm/v/s at the tile's first element in the arenas.
template <int VEC, int OP, bool BF16, int NT, bool FULL, bool EXT>
__device__ __forceinline__ void apply_tile(const ApplyArgs &a, void *xu, const void *gu, float *xm,
                                           float *v, float *s, const float4 (&zt)[VEC], float wd,
                                           uint32_t count, uint32_t lane, float neg_lr, float alpha)
{
    constexpr bool NEED_G = (OP == OP_STEP || OP == OP_STEP_MERGE);
    constexpr bool NEED_V = NEED_G;
    constexpr bool NEED_X = (OP != OP_INIT);
    constexpr bool NEED_S = (OP == OP_MERGE || OP == OP_STEP_MERGE);
    constexpr bool WRITE_X = (OP != OP_SNAPSHOT);
    constexpr bool WRITE_V = NEED_V || OP == OP_INIT;
    float *xf = BF16 ? xm : static_cast<float *>(xu);          // where the fp32 model lives
    uint16_t *x16 = static_cast<uint16_t *>(xu);
    const float *gf = static_cast<const float *>(gu);
    const uint16_t *g16 = static_cast<const uint16_t *>(gu);
    const bool write_s = (OP == OP_SNAPSHOT) || (NEED_S && a.resnap);

    if constexpr (FULL) {
        float4 x[VEC], vv[VEC], g[VEC], ss[VEC];
        // all loads first: up to 4*VEC independent 128-bit loads in flight per lane
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            const uint32_t e = j * 256u + lane * 4u;
            if constexpr (NEED_G) g[j] = BF16 ? widen4(ld2<NT>(g16 + e)) : ld4<NT>(gf + e);
            if constexpr (NEED_X) x[j] = ld4<NT>(xf + e);
            if constexpr (OP == OP_INIT) x[j] = widen4(ld2<NT>(x16 + e));
            if constexpr (NEED_V) vv[j] = ld4<NT>(v + e);
            if constexpr (NEED_S) ss[j] = ld4<NT>(s + e);
        }
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            const uint32_t e = j * 256u + lane * 4u;
            if constexpr (NEED_G)
                LASGD_FOR4(step_elem(comp(x[j], c), comp(vv[j], c), compv(g[j], c), wd, a.mu,
                                     neg_lr, a.nesterov);)
            if constexpr (NEED_S) {
                if constexpr (EXT)
                    LASGD_FOR4(comp(x[j], c) = merge_elem_elastic(compv(x[j], c), compv(ss[j], c), compv(zt[j], c), alpha);)
                else
                    LASGD_FOR4(comp(x[j], c) = merge_elem(compv(x[j], c), compv(ss[j], c), compv(zt[j], c));)
            }
            if constexpr (OP == OP_INIT) vv[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if constexpr (WRITE_V) st4<NT>(v + e, vv[j]);
            if constexpr (WRITE_X) {
                st4<NT>(xf + e, x[j]);
                if constexpr (BF16 && OP != OP_INIT) st2<NT>(x16 + e, round4(x[j]));
            }
            if (write_s) st4<NT>(s + e, x[j]);
        }
    } else {
        // ragged tile: same arithmetic, element by element where a 128-bit
        // access would cross the end of the tensor
        // (fully unrolled over j so that the z registers are never indexed at run time)
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            const uint32_t e0 = j * 256u + lane * 4u;
            const uint32_t n = (e0 >= count) ? 0u : (count - e0 < 4u) ? count - e0 : 4u;
            for (uint32_t i = 0; i < n; ++i) {
                const uint32_t e = e0 + i;
                float xe = 0.f, ve = 0.f, ge = 0.f, se = 0.f;
                if constexpr (NEED_G) ge = BF16 ? bf16_widen(g16[e]) : gf[e];
                if constexpr (NEED_X) xe = xf[e];
                if constexpr (OP == OP_INIT) xe = bf16_widen(x16[e]);
                if constexpr (NEED_V) ve = v[e];
                if constexpr (NEED_S) se = s[e];
                if constexpr (NEED_G) step_elem(xe, ve, ge, wd, a.mu, neg_lr, a.nesterov);
                if constexpr (NEED_S)
                    xe = EXT ? merge_elem_elastic(xe, se, compv(zt[j], (int)i), alpha)
                             : merge_elem(xe, se, compv(zt[j], (int)i));
                if constexpr (WRITE_V) v[e] = ve;
                if constexpr (WRITE_X) {
                    xf[e] = xe;
                    if constexpr (BF16 && OP != OP_INIT) x16[e] = (uint16_t)bf16_round(xe);
                }
                if (write_s) s[e] = xe;
            }
        }
    }
}

// Multi-tensor apply.  Work item = (tile, group of kper replicas); one wave
// per item, items strided over the grid.  All table reads are wave-uniform.
// The waves of a workgroup are independent (no LDS, no barrier), so the
// workgroup size (64, 128 or 256 threads) is purely a dispatch-granularity knob.
template <int VEC, int OP, bool BF16, int NT, bool EXT>
__device__ __forceinline__ void apply_body(const ApplyArgs &a, const ExtArgs *xa)
{
    constexpr bool NEED_Z = (OP == OP_MERGE || OP == OP_STEP_MERGE);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wpb = blockDim.x >> 6;                  // independent waves per workgroup
    const uint32_t wave0 = __builtin_amdgcn_readfirstlane(blockIdx.x * wpb + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * wpb;
    for (uint32_t item = wave0; item < a.nitems; item += nwaves) {
        // Item order: tiles are taken in chunks of a.chunk; inside a chunk the items run
        // replica group by replica group, so that each replica's arrays are swept in
        // contiguous runs of a.chunk tiles while the chunk's z tiles are reused K times
        // within a short window (chunk = 1: the replicas of one tile are adjacent;
        // chunk = ntiles: one replica after the other).  Workgroups go to the eight
        // XCDs round-robin, each with its own L2: when a chunk is a multiple of eight
        // workgroups long, tile j of every replica lands on the same XCD, so only the
        // first replica's request for a z tile misses that L2.  The last, shorter chunk is
        // padded with idle items to such a multiple for the same reason.
        uint32_t tile, kg;
        if (item < a.full_items) {
            const uint32_t per = a.chunk * a.kgroups;
            const uint32_t ch = item / per;
            const uint32_t r = item - ch * per;
            kg = r / a.chunk;
            tile = ch * a.chunk + (r - kg * a.chunk);
        } else {
            const uint32_t r = item - a.full_items;
            kg = r / a.tail_stride;
            const uint32_t i = r - kg * a.tail_stride;
            if (i >= a.tail_chunk) continue;                    // padding item
            tile = a.tail_first + i;
        }
        const Tile t = load_tile(a.tiles + tile);
        const bool full = (t.count == 256u * VEC);
        float4 zt[VEC];
        if constexpr (NEED_Z) {
            const float *zp = a.z + t.aoff;
            if (full) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) zt[j] = *reinterpret_cast<const float4 *>(zp + j * 256u + lane * 4u);
            } else {
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    const uint32_t e0 = j * 256u + lane * 4u;
                    zt[j].x = (e0 + 0u < t.count) ? zp[e0 + 0u] : 0.f;
                    zt[j].y = (e0 + 1u < t.count) ? zp[e0 + 1u] : 0.f;
                    zt[j].z = (e0 + 2u < t.count) ? zp[e0 + 2u] : 0.f;
                    zt[j].w = (e0 + 3u < t.count) ? zp[e0 + 3u] : 0.f;
                }
            }
        }
        const uint32_t k0 = kg * a.kper;
        const uint32_t k1 = (k0 + a.kper < a.K) ? k0 + a.kper : a.K;
        for (uint32_t k = k0; k < k1; ++k) {
            const size_t pi = (size_t)k * a.n_tensors + t.tensor;
            const size_t esz = BF16 ? 2 : 4;
            char *xu = load_ptr(a.xptr, pi) + t.toff * esz;
            const char *gu = nullptr;
            if constexpr (OP == OP_STEP || OP == OP_STEP_MERGE)
                gu = load_ptr(a.gptr, pi) + t.toff * esz;
            const size_t ao = (size_t)k * a.npad + t.aoff;
            float *xm = BF16 ? a.x32 + ao : nullptr;
#define LASGD_TILE(OPX, NLR, AL)                                                                             \
    do {                                                                                                     \
        if (full) apply_tile<VEC, OPX, BF16, NT, true, EXT>(a, xu, gu, xm, a.v + ao, a.s + ao, zt, t.wd, t.count, lane, NLR, AL); \
        else apply_tile<VEC, OPX, BF16, NT, false, EXT>(a, xu, gu, xm, a.v + ao, a.s + ao, zt, t.wd, t.count, lane, NLR, AL);     \
    } while (0)
            if constexpr (!EXT) {
                LASGD_TILE(OP, a.neg_lr, 1.0f);
            } else {
                // a replica may take the local update, the global update, both or neither
                const bool in_step = (xa->step_mask >> k) & 1ull;
                const bool in_merge = (xa->merge_mask >> k) & 1ull;
                const float nlr = xa->neg_lr_k[k];
                if constexpr (OP == OP_STEP_MERGE) {
                    if (in_step && in_merge) LASGD_TILE(OP_STEP_MERGE, nlr, xa->alpha);
                    else if (in_step) LASGD_TILE(OP_STEP, nlr, 1.0f);
                    else if (in_merge) LASGD_TILE(OP_MERGE, 0.0f, xa->alpha);
                } else if constexpr (OP == OP_MERGE) {
                    if (in_merge) LASGD_TILE(OP_MERGE, 0.0f, xa->alpha);
                } else {
                    if (in_step) LASGD_TILE(OP, nlr, 1.0f);
                }
            }
#undef LASGD_TILE
        }
    }
}

template <int VEC, int OP, bool BF16, int NT>
__global__ __launch_bounds__(256) void apply_kernel(const ApplyArgs a)
{
    apply_body<VEC, OP, BF16, NT, false>(a, nullptr);
}

template <int VEC, int OP, bool BF16, int NT>
__global__ __launch_bounds__(256) void apply_ext_kernel(const ApplyArgs a, const ExtArgs xa)
{
    apply_body<VEC, OP, BF16, NT, true>(a, &xa);
}

// ---- the mean (Sec. 3, Eq. 8) -----------------------------------------------
// z[e] = (1/K) sum_k s[k][e], fp64 accumulation in replica order, one rounding.
// The arenas are contiguous and padded with zeros, so this is a flat pass.
// EXT variants: the mean runs over a list of participants (partial All-Reduce,
// Sec. 6; the divisor is their number) and may be blended into the previous
// centre, z = (1-beta) z + beta mean (Sec. 3, Eq. 5).
struct AvgArgs {
    const float *s;
    float *z;
    uint64_t npad;      // elements per replica, multiple of 4
    uint64_t nvec;      // npad / 4
    uint32_t K;         // replicas summed (participants in the EXT variants)
    int32_t use_mul;    // K is a power of two: multiply by the exact reciprocal
    double inv_k, k_as_double;
    int32_t elastic;    // EXT: blend with the previous centre
    double beta, one_minus_beta;
    uint8_t idx[64];    // EXT: the participants, ascending
};

template <bool EXT> __device__ __forceinline__ uint32_t replica_of(const AvgArgs &a, uint32_t j)
{
    if constexpr (EXT) return a.idx[j];
    else return j;
}

template <bool EXT> __device__ __forceinline__ float finish_mean(double acc, float z_old, const AvgArgs &a)
{
    const double mean = a.use_mul ? acc * a.inv_k : acc / a.k_as_double;
    if constexpr (EXT) {
        if (a.elastic) {
            const double keep = a.one_minus_beta * (double)z_old;
            const double pull = a.beta * mean;
            return (float)(keep + pull);
        }
    }
    return (float)mean;
}

#define LASGD_ACC4(r)                                                                          \
    do { a0 += (double)(r).x; a1 += (double)(r).y; a2 += (double)(r).z; a3 += (double)(r).w; } while (0)

// SPLIT == 1: every lane owns one 128-bit column and walks all K replicas,
// eight loads in flight at a time.
template <int NT, bool EXT>
__global__ __launch_bounds__(256) void average_kernel(const AvgArgs a)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.nvec; i += stride) {
        const float *p = a.s + i * 4u;
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
        uint32_t k = 0;
        for (; k + 8u <= a.K; k += 8u) {
            float4 r[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) r[u] = ld4<NT>(p + (uint64_t)replica_of<EXT>(a, k + u) * a.npad);
#pragma unroll
            for (int u = 0; u < 8; ++u) LASGD_ACC4(r[u]);
        }
        if (k + 4u <= a.K) {
            float4 r[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) r[u] = ld4<NT>(p + (uint64_t)replica_of<EXT>(a, k + u) * a.npad);
#pragma unroll
            for (int u = 0; u < 4; ++u) LASGD_ACC4(r[u]);
            k += 4u;
        }
        for (; k < a.K; ++k) {
            float4 r = ld4<NT>(p + (uint64_t)replica_of<EXT>(a, k) * a.npad);
            LASGD_ACC4(r);
        }
        float4 zo = make_float4(0.f, 0.f, 0.f, 0.f);
        if constexpr (EXT) {
            if (a.elastic) zo = *reinterpret_cast<const float4 *>(a.z + i * 4u);
        }
        float4 out = make_float4(finish_mean<EXT>(a0, zo.x, a), finish_mean<EXT>(a1, zo.y, a),
                                 finish_mean<EXT>(a2, zo.z, a), finish_mean<EXT>(a3, zo.w, a));
        st4<NT>(a.z + i * 4u, out);
    }
}

// SPLIT in {2, 4}: the K replicas of one 256/SPLIT-column tile are divided
// among SPLIT groups of waves; each group sums a contiguous range of replicas
// in fp64, the partial sums meet in LDS and are added in group order.  More
// independent load streams per column for large K; the result can differ from
// the in-order sum only by fp64 rounding, i.e. in fp32 only at double-rounding ties.
template <int SPLIT, int NT, bool EXT>
__global__ __launch_bounds__(256) void average_split_kernel(const AvgArgs a)
{
    constexpr uint32_t COLS = 256u / SPLIT;             // 128-bit columns per workgroup pass
    __shared__ double part[SPLIT][COLS][4];
    const uint32_t g = threadIdx.x / COLS;              // which replica range
    const uint32_t c = threadIdx.x % COLS;
    const uint32_t kb = (uint32_t)(((uint64_t)a.K * g) / SPLIT);
    const uint32_t ke = (uint32_t)(((uint64_t)a.K * (g + 1u)) / SPLIT);
    const uint64_t ntile = (a.nvec + COLS - 1u) / COLS;
    for (uint64_t tile = blockIdx.x; tile < ntile; tile += gridDim.x) {
        const uint64_t i = tile * COLS + c;
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
        if (i < a.nvec) {
            const float *p = a.s + i * 4u;
            uint32_t k = kb;
            for (; k + 4u <= ke; k += 4u) {
                float4 r[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) r[u] = ld4<NT>(p + (uint64_t)replica_of<EXT>(a, k + u) * a.npad);
#pragma unroll
                for (int u = 0; u < 4; ++u) LASGD_ACC4(r[u]);
            }
            for (; k < ke; ++k) {
                float4 r = ld4<NT>(p + (uint64_t)replica_of<EXT>(a, k) * a.npad);
                LASGD_ACC4(r);
            }
        }
        part[g][c][0] = a0; part[g][c][1] = a1; part[g][c][2] = a2; part[g][c][3] = a3;
        __syncthreads();
        // 256 threads finish COLS*4 = 1024/SPLIT elements: 4/SPLIT each, consecutive
        constexpr uint32_t PER = 4u / SPLIT;             // 2 or 1
        const uint32_t e0 = threadIdx.x * PER;           // element within the tile
        const uint64_t ebase = tile * COLS * 4u + e0;
        const bool inside = ebase + PER <= a.npad;
        float outv[PER];
#pragma unroll
        for (uint32_t q = 0; q < PER; ++q) {
            const uint32_t e = e0 + q;
            double acc = 0.0;
#pragma unroll
            for (int gg = 0; gg < SPLIT; ++gg) acc += part[gg][e >> 2][e & 3u];
            float zo = 0.f;
            if constexpr (EXT) {
                if (a.elastic && inside) zo = a.z[ebase + q];
            }
            outv[q] = finish_mean<EXT>(acc, zo, a);
        }
        if (inside) {
            if constexpr (PER == 2) *reinterpret_cast<float2 *>(a.z + ebase) = make_float2(outv[0], outv[PER - 1]);
            else a.z[ebase] = outv[0];
        }
        __syncthreads();
    }
}

// ---- replica-group kernels ----------------------------------------------------
// Two operations need all K replicas of an element at once: the mean gradient of
// the SGD All-Reduce comparator, and the next mean z when it is computed in the
// same pass as the global update.  Both use one workgroup per tile with one wave
// per replica (wave w owns replicas w, w + W, ... when K exceeds the W = 16 waves
// a workgroup can hold).  Every wave streams its own replica's arrays exactly as
// the one-wave-per-(tile, replica) kernels do, the K values of each element meet
// in LDS as fp32 (exact), and the sum runs in fp64 in replica order, so the result
// is bit-identical to the in-order mean.  The tile is processed in rows of 256
// elements; LDS holds one row per replica (K KiB).
constexpr uint32_t kGroupWaves = 16;

// Elements [e0, e0+4) of one row for this lane; n = how many of them exist.
template <int NT, bool FULL> __device__ __forceinline__ float4 row_ld(const float *p, uint32_t e0, uint32_t n)
{
    if (FULL || n == 4u) return ld4<NT>(p + e0);
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (n > 0u) r.x = p[e0];
    if (n > 1u) r.y = p[e0 + 1u];
    if (n > 2u) r.z = p[e0 + 2u];
    return r;
}
template <int NT, bool FULL> __device__ __forceinline__ float4 row_ld16(const uint16_t *p, uint32_t e0, uint32_t n)
{
    if (FULL || n == 4u) return widen4(ld2<NT>(p + e0));
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (n > 0u) r.x = bf16_widen(p[e0]);
    if (n > 1u) r.y = bf16_widen(p[e0 + 1u]);
    if (n > 2u) r.z = bf16_widen(p[e0 + 2u]);
    return r;
}
template <int NT, bool FULL> __device__ __forceinline__ void row_st(float *p, uint32_t e0, uint32_t n, float4 a)
{
    if (FULL || n == 4u) { st4<NT>(p + e0, a); return; }
    if (n > 0u) p[e0] = a.x;
    if (n > 1u) p[e0 + 1u] = a.y;
    if (n > 2u) p[e0 + 2u] = a.z;
}
template <int NT, bool FULL> __device__ __forceinline__ void row_st16(uint16_t *p, uint32_t e0, uint32_t n, float4 a)
{
    if (FULL || n == 4u) { st2<NT>(p + e0, round4(a)); return; }
    if (n > 0u) p[e0] = (uint16_t)bf16_round(a.x);
    if (n > 1u) p[e0 + 1u] = (uint16_t)bf16_round(a.y);
    if (n > 2u) p[e0 + 2u] = (uint16_t)bf16_round(a.z);
}

__device__ __forceinline__ float group_mean_of(double acc, const ApplyArgs &a)
{
    return (float)(a.use_mul ? acc * a.inv_k : acc / a.k_as_double);
}

// Where replica k keeps one tile: the fp32 model (the caller's buffer, or the master
// copy for bf16 storage), the caller's 16-bit parameters and gradient, v and s.
template <bool BF16> struct ReplicaTile {
    float *xf, *v, *s;
    uint16_t *x16;
    const void *g;
};
template <bool BF16>
__device__ __forceinline__ ReplicaTile<BF16> replica_tile(const ApplyArgs &a, const Tile &t, uint32_t k)
{
    constexpr size_t ESZ = BF16 ? 2 : 4;
    const size_t pi = (size_t)k * a.n_tensors + t.tensor;
    const size_t ao = (size_t)k * a.npad + t.aoff;
    char *xu = load_ptr(a.xptr, pi) + t.toff * ESZ;
    ReplicaTile<BF16> r;
    r.xf = BF16 ? a.x32 + ao : reinterpret_cast<float *>(xu);
    r.x16 = reinterpret_cast<uint16_t *>(xu);
    r.v = a.v + ao;
    r.s = a.s + ao;
    r.g = load_ptr(a.gptr, pi) + t.toff * ESZ;
    return r;
}
template <bool BF16, int NT, bool FULL>
__device__ __forceinline__ float4 row_ld_grad(const void *g, uint32_t e0, uint32_t n)
{
    if constexpr (BF16) return row_ld16<NT, FULL>(static_cast<const uint16_t *>(g), e0, n);
    else return row_ld<NT, FULL>(static_cast<const float *>(g), e0, n);
}

// A wave owns replicas w + q*W, q = 0, 1, ...; it takes them R at a time ("pass").
// A wave whose pass runs past K re-reads replica K-1 and keeps nothing of it, so
// that the loads of a pass stay free of branches.

// SGD All-Reduce comparator (Sec. 2; "SGD-AR" of Table 1), one row of a tile:
// the K gradients are averaged (fp64 in replica order, one rounding to fp32) and
// every replica takes the local update with that mean gradient.  Same 20 bytes
// per replica-parameter as a local step.
template <int R, bool BF16, int NT, bool FULL>
__device__ __forceinline__ void sgd_ar_row(const ApplyArgs &a, const Tile &t, float *lds, uint32_t row,
                                           uint32_t w, uint32_t W, uint32_t passes, uint32_t lane)
{
    const uint32_t e0 = row * 256u + lane * 4u;
    const uint32_t n = FULL ? 4u : (e0 >= t.count) ? 0u : (t.count - e0 < 4u) ? t.count - e0 : 4u;
    // first pass: the model loads are issued with the gradient loads, ahead of the exchange
    float4 x[R], v[R];
    ReplicaTile<BF16> rt[R];
    bool mine[R];
    {
        float4 g[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t kw = w + (uint32_t)r * W;
            mine[r] = kw < a.K;
            rt[r] = replica_tile<BF16>(a, t, mine[r] ? kw : a.K - 1u);
            g[r] = row_ld_grad<BF16, NT, FULL>(rt[r].g, e0, n);
            x[r] = row_ld<NT, FULL>(rt[r].xf, e0, n);
            v[r] = row_ld<NT, FULL>(rt[r].v, e0, n);
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (mine[r]) *reinterpret_cast<float4 *>(lds + (size_t)(w + (uint32_t)r * W) * 256u + lane * 4u) = g[r];
    }
    for (uint32_t p = 1; p < passes; ++p) {
        float4 g[R];
        uint32_t kw[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            kw[r] = w + (p * R + (uint32_t)r) * W;
            const ReplicaTile<BF16> q = replica_tile<BF16>(a, t, kw[r] < a.K ? kw[r] : a.K - 1u);
            g[r] = row_ld_grad<BF16, NT, FULL>(q.g, e0, n);
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (kw[r] < a.K) *reinterpret_cast<float4 *>(lds + (size_t)kw[r] * 256u + lane * 4u) = g[r];
    }
    __syncthreads();
    // every wave sums the row itself: handing the sum to a few waves and passing the result
    // round through LDS costs a second barrier and measured slower than the repeated fp64 adds
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    for (uint32_t k = 0; k < a.K; ++k) {
        const float4 q = *reinterpret_cast<const float4 *>(lds + (size_t)k * 256u + lane * 4u);
        LASGD_ACC4(q);
    }
    const float4 gbar = make_float4(group_mean_of(a0, a), group_mean_of(a1, a), group_mean_of(a2, a), group_mean_of(a3, a));
#pragma unroll
    for (int r = 0; r < R; ++r) {
        LASGD_FOR4(step_elem(comp(x[r], c), comp(v[r], c), compv(gbar, c), t.wd, a.mu, a.neg_lr, a.nesterov);)
        if (mine[r]) {
            row_st<NT, FULL>(rt[r].v, e0, n, v[r]);
            row_st<NT, FULL>(rt[r].xf, e0, n, x[r]);
            if constexpr (BF16) row_st16<NT, FULL>(rt[r].x16, e0, n, x[r]);
        }
    }
    for (uint32_t p = 1; p < passes; ++p) {
        ReplicaTile<BF16> q[R];
        float4 xx[R], vv[R];
        bool ok[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t kw = w + (p * R + (uint32_t)r) * W;
            ok[r] = kw < a.K;
            q[r] = replica_tile<BF16>(a, t, ok[r] ? kw : a.K - 1u);
            xx[r] = row_ld<NT, FULL>(q[r].xf, e0, n);
            vv[r] = row_ld<NT, FULL>(q[r].v, e0, n);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            LASGD_FOR4(step_elem(comp(xx[r], c), comp(vv[r], c), compv(gbar, c), t.wd, a.mu, a.neg_lr, a.nesterov);)
            if (ok[r]) {
                row_st<NT, FULL>(q[r].v, e0, n, vv[r]);
                row_st<NT, FULL>(q[r].xf, e0, n, xx[r]);
                if constexpr (BF16) row_st16<NT, FULL>(q[r].x16, e0, n, xx[r]);
            }
        }
    }
    __syncthreads();                 // the next row reuses the LDS buffer
}

template <int R, bool BF16, int NT>
__global__ __launch_bounds__(1024) void sgd_ar_kernel(const ApplyArgs a, const uint32_t passes)
{
    extern __shared__ float lds[];                        // [K][256]
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t W = blockDim.x >> 6;
    for (uint32_t tile = blockIdx.x; tile < a.ntiles; tile += gridDim.x) {
        const Tile t = load_tile(a.tiles + tile);
        const uint32_t rows = (t.count + 255u) >> 8;
        for (uint32_t row = 0; row < rows; ++row) {
            if (t.count - row * 256u >= 256u) sgd_ar_row<R, BF16, NT, true>(a, t, lds, row, w, W, passes, lane);
            else sgd_ar_row<R, BF16, NT, false>(a, t, lds, row, w, W, passes, lane);
        }
    }
}

// Steps 7 and 9a-c of Algorithm 1 and the next All-Reduce (Sec. 3, Eq. 8) in one
// pass: every replica takes its local update, then the global update with the
// pending z, re-sends (s <- x), and the tile's next z -- the mean of the models
// just sent -- is written over the old one.  Only this workgroup touches the
// tile's z, and all its waves have used the old values before the barrier.
// Same roundings as step_merge followed by the in-order mean.
template <int R, bool BF16, int NT, bool FULL>
__device__ __forceinline__ void step_merge_mean_row(const ApplyArgs &a, const Tile &t, float *lds, uint32_t row,
                                                    uint32_t w, uint32_t W, uint32_t passes, uint32_t lane)
{
    const uint32_t e0 = row * 256u + lane * 4u;
    const uint32_t n = FULL ? 4u : (e0 >= t.count) ? 0u : (t.count - e0 < 4u) ? t.count - e0 : 4u;
    const float4 z = row_ld<0, FULL>(a.z + t.aoff, e0, n);         // shared by the K waves: cacheable
    for (uint32_t p = 0; p < passes; ++p) {
        ReplicaTile<BF16> q[R];
        float4 x[R], v[R], g[R], ss[R];
        uint32_t kw[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            kw[r] = w + (p * R + (uint32_t)r) * W;
            q[r] = replica_tile<BF16>(a, t, kw[r] < a.K ? kw[r] : a.K - 1u);
            g[r] = row_ld_grad<BF16, NT, FULL>(q[r].g, e0, n);
            x[r] = row_ld<NT, FULL>(q[r].xf, e0, n);
            v[r] = row_ld<NT, FULL>(q[r].v, e0, n);
            ss[r] = row_ld<NT, FULL>(q[r].s, e0, n);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            LASGD_FOR4(step_elem(comp(x[r], c), comp(v[r], c), compv(g[r], c), t.wd, a.mu, a.neg_lr, a.nesterov);)
            LASGD_FOR4(comp(x[r], c) = merge_elem(compv(x[r], c), compv(ss[r], c), compv(z, c));)
            if (kw[r] < a.K) {
                row_st<NT, FULL>(q[r].v, e0, n, v[r]);
                row_st<NT, FULL>(q[r].xf, e0, n, x[r]);
                if constexpr (BF16) row_st16<NT, FULL>(q[r].x16, e0, n, x[r]);
                row_st<NT, FULL>(q[r].s, e0, n, x[r]);
                *reinterpret_cast<float4 *>(lds + (size_t)kw[r] * 256u + lane * 4u) = x[r];
            }
        }
    }
    __syncthreads();
    // up to four waves finish the row's mean, one element per thread and turn
    const uint32_t fin = (W < 4u ? W : 4u) * 64u;
    if (threadIdx.x < fin) {
        for (uint32_t c = threadIdx.x; c < 256u; c += fin) {
            const uint32_t e = row * 256u + c;
            if (FULL || e < t.count) {
                double acc = 0.0;
                for (uint32_t k = 0; k < a.K; ++k) acc += (double)lds[(size_t)k * 256u + c];
                a.z[t.aoff + e] = group_mean_of(acc, a);
            }
        }
    }
    __syncthreads();
}

template <int R, bool BF16, int NT>
__global__ __launch_bounds__(1024) void step_merge_mean_kernel(const ApplyArgs a, const uint32_t passes)
{
    extern __shared__ float lds[];                        // [K][256]
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t W = blockDim.x >> 6;
    for (uint32_t tile = blockIdx.x; tile < a.ntiles; tile += gridDim.x) {
        const Tile t = load_tile(a.tiles + tile);
        const uint32_t rows = (t.count + 255u) >> 8;
        for (uint32_t row = 0; row < rows; ++row) {
            if (t.count - row * 256u >= 256u) step_merge_mean_row<R, BF16, NT, true>(a, t, lds, row, w, W, passes, lane);
            else step_merge_mean_row<R, BF16, NT, false>(a, t, lds, row, w, W, passes, lane);
        }
    }
}

// Debugging aid for the two-stream protocol: fill z with NaN.
__global__ __launch_bounds__(256) void poison_kernel(float *z, uint64_t n)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) z[i] = __uint_as_float(0x7fc00000u);
}

// ---- context-free global update on flat fp32 vectors -------------------------
// For callers that hold no context and may not allocate: the mean (Sec. 3,
// Eq. 8) of K sent models goes to a buffer the host names, and the global
// update (Algorithm 1 step 9a-c) reads it back.  Same arithmetic and rounding
// order as the kernels above; replica pointers travel in the kernel arguments.
struct FlatArgs {
    float *x[64];       // local models, n elements each
    float *s[64];       // sent models
    float *z;           // the mean, n elements (library scratch)
    uint64_t n;
    uint64_t nvec;      // n / 4
    uint32_t K;
    int32_t use_mul;    // K is a power of two: multiply by the exact reciprocal
    double inv_k, k_as_double;
    int32_t resnap;
};

__device__ __forceinline__ float flat_mean_of(double acc, const FlatArgs &a)
{
    return (float)(a.use_mul ? acc * a.inv_k : acc / a.k_as_double);
}

__global__ __launch_bounds__(256) void flat_mean_kernel(const FlatArgs a)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (uint64_t i = tid; i < a.nvec; i += stride) {
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
        for (uint32_t k = 0; k < a.K; ++k) {
            const float4 r = ld4<0>(a.s[k] + i * 4u);
            LASGD_ACC4(r);
        }
        st4<0>(a.z + i * 4u, make_float4(flat_mean_of(a0, a), flat_mean_of(a1, a), flat_mean_of(a2, a), flat_mean_of(a3, a)));
    }
    // the last n % 4 elements, one thread each
    const uint64_t e = a.nvec * 4u + tid;
    if (e < a.n) {
        double acc = 0.0;
        for (uint32_t k = 0; k < a.K; ++k) acc += (double)a.s[k][e];
        a.z[e] = flat_mean_of(acc, a);
    }
}

// grid.y = replica; grid.x strides over the 128-bit vectors of that replica
__global__ __launch_bounds__(256) void flat_merge_kernel(const FlatArgs a)
{
    const uint32_t k = blockIdx.y;
    float *x = a.x[k], *s = a.s[k];
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (uint64_t i = tid; i < a.nvec; i += stride) {
        float4 xv = ld4<0>(x + i * 4u);
        const float4 sv = ld4<0>(s + i * 4u);
        const float4 zv = ld4<0>(a.z + i * 4u);
        LASGD_FOR4(comp(xv, c) = merge_elem(compv(xv, c), compv(sv, c), compv(zv, c));)
        st4<0>(x + i * 4u, xv);
        if (a.resnap) st4<0>(s + i * 4u, xv);
    }
    const uint64_t e = a.nvec * 4u + tid;
    if (e < a.n) {
        const float xn = merge_elem(x[e], s[e], a.z[e]);
        x[e] = xn;
        if (a.resnap) s[e] = xn;
    }
}

} // namespace lasgd
