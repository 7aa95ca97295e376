// Host side of the LASGD update library: context, validation, state machine,
// descriptor tables, launches.  The C ABI is declared in include/lasgd.h.
//
// Stream protocol (single-GPU image of "the All-Reduce runs while the node
// keeps computing", Sec. 4):
//   main stream:  local_step ... snapshot/merge --evA--> ...        wait evZ, merge
//   side stream:                          wait evA, average --evZ-->
// evA orders the side stream's reads of s after the main stream's writes;
// evZ orders the main stream's reads of z after the side stream's writes.
// The state machine refuses call orders in which s or z could be overwritten
// while the other stream may still read them.
#include "lasgd_kernels.hip.h"
#include "../../include/lasgd.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace lasgd;

namespace {

constexpr int kMaxK = 64;
// Elements.  Every tensor starts on 1 KiB inside a replica's slab, so that each 256-element tile is one aligned
// KiB: tiles that start 256 or 512 bytes off such a boundary stream 3-5 % slower on MI355X.
constexpr uint64_t kArenaAlign = 256;
constexpr uint64_t kMaxNpad = (1ull << 31) - (1ull << 20); // tile offsets stay far inside 32-bit element counts

thread_local std::string g_create_error;

} // namespace

struct lasgd_ctx {
    int32_t K = 0, n_tensors = 0;
    lasgd_dtype storage = LASGD_F32;
    float mu = 0.f, wd_scalar = 0.f;
    int32_t nesterov = 0;
    std::vector<int64_t> numel;
    std::vector<float> wd;
    std::vector<uint64_t> aoff;      // arena offset of each tensor (elements)
    uint64_t npad = 0, ntotal = 0;
    hipStream_t main = nullptr, side = nullptr;
    hipEvent_t evA = nullptr, evZ = nullptr;
    int device = 0;

    // device memory (one allocation, carved up)
    char *arena = nullptr;
    float *v = nullptr, *s = nullptr, *z = nullptr, *x32 = nullptr;
    Tile *tiles = nullptr;           // the table for the current tile size (one of tiles_by_vec)
    uint32_t ntiles = 0;
    // one table per tile size ever used (vec = 1, 2, 4), kept until destroy: a graph captured
    // under one tile size still points at its table after the tile size has been changed
    Tile *tiles_by_vec[3] = {nullptr, nullptr, nullptr};
    uint32_t ntiles_by_vec[3] = {0, 0, 0};
    void **xptr = nullptr, **gptr = nullptr;     // device tables [K*n_tensors]
    std::vector<void *> h_xptr, h_gptr;
    std::vector<char> bound;
    int32_t n_bound = 0;

    // protocol state (bit k = replica k)
    bool master_ready = false;   // bf16: master copy initialised
    uint64_t all = 0;            // every replica
    uint64_t snap_mask = 0;      // s[k] holds a model that may be averaged next
    uint64_t pending_mask = 0;   // participants of the launched mean that have not merged yet
    bool avg_ever = false;
    bool avg_in_graph = false;   // the last mean was recorded into a graph, not executed: evZ says nothing about it
    bool z_on_main = false;      // the pending mean was enqueued on the main stream: stream order already puts it first
    bool center_valid = false;   // z has been computed at least once
    float alpha = 1.f, beta = 1.f;   // elastic coefficients (Sec. 3, Eq. 5-6); 1, 1 = Algorithm 1

    lasgd_tuning tune{};
    std::string err;
};

namespace {

lasgd_status fail(lasgd_ctx *ctx, lasgd_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    try {
        if (ctx) ctx->err = buf;
        else g_create_error = buf;
    } catch (...) {       // the message is lost, the status is not
    }
    return st;
}

#define LASGD_HIP(ctx, call)                                                                   \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess) {                                                                \
            (void)hipGetLastError(); /* reported here; do not leave it for the next HIP user */ \
            return fail(ctx, e_ == hipErrorOutOfMemory ? LASGD_ERR_ALLOC : LASGD_ERR_HIP,      \
                        "%s failed: %s", #call, hipGetErrorString(e_));                        \
        }                                                                                      \
    } while (0)

uint64_t round_up(uint64_t a, uint64_t b) { return (a + b - 1) / b * b; }

bool is_pow2(uint32_t k) { return k && !(k & (k - 1)); }

// Build (on the host) the tile list for 256*vec-element tiles.
std::vector<Tile> build_tiles(const lasgd_ctx &c, int vec)
{
    std::vector<Tile> t;
    const uint64_t T = 256ull * vec;
    for (int32_t i = 0; i < c.n_tensors; ++i) {
        const uint64_t n = (uint64_t)c.numel[i];
        for (uint64_t o = 0; o < n; o += T) {
            Tile d{};
            d.toff = o;
            d.aoff = c.aoff[i] + o;
            d.tensor = (uint32_t)i;
            d.count = (uint32_t)((n - o < T) ? n - o : T);
            d.wd = c.wd[i];
            t.push_back(d);
        }
    }
    return t;
}

lasgd_status upload_tiles(lasgd_ctx *c, int vec)
{
    const int slot = vec == 1 ? 0 : vec == 2 ? 1 : 2;
    if (!c->tiles_by_vec[slot]) {
        std::vector<Tile> t = build_tiles(*c, vec);
        if (t.size() > 0x7fffffffull / kMaxK) return fail(c, LASGD_ERR_UNSUPPORTED, "too many tiles (%zu)", t.size());
        Tile *d = nullptr;
        LASGD_HIP(c, hipMalloc(&d, t.size() * sizeof(Tile)));
        hipError_t e = hipMemcpy(d, t.data(), t.size() * sizeof(Tile), hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipFree(d);
            (void)hipGetLastError();
            return fail(c, LASGD_ERR_HIP, "tile table upload failed: %s", hipGetErrorString(e));
        }
        c->tiles_by_vec[slot] = d;
        c->ntiles_by_vec[slot] = (uint32_t)t.size();
    }
    c->tiles = c->tiles_by_vec[slot];
    c->ntiles = c->ntiles_by_vec[slot];
    return LASGD_OK;
}

// Defaults from sweeps on MI355X over the five benchmark workloads: the finest
// tile (one 128-bit vector per lane), one wave per (tile, replica), a grid that
// covers all items in one-wave workgroups (the waves are independent, and
// single-wave groups dispatch and retire with the least friction), and the
// streaming hint on every access except z once the state no longer fits the
// 256 MB memory-side cache.  A local step sweeps one replica after the other
// (the longest contiguous runs); merges take the tiles in chunks of 8192 (8 MB
// of z per chunk, 1 MB per XCD) so that the chunk's z is still in L2 when the
// next replica needs it.  The split mean (256-thread workgroups with LDS) wins
// from K = 8 upwards; next to one-wave workgroups of a local step it is
// dispatched sparingly, which keeps the step fast, and split 2 still ends well
// before the next global update at m = 4 (split 4 trickles until just before it).
lasgd_tuning default_tuning(const lasgd_ctx &c)
{
    lasgd_tuning t{};
    t.vec = 1;
    t.kper_step = 1;
    t.kper_merge = 1;
    t.max_blocks = -1;
    t.avg_split = c.K >= 8 ? 2 : 1;
    t.avg_max_blocks = -1;
    t.nontemporal = ((uint64_t)c.K * c.npad * sizeof(float) >= (128ull << 20)) ? 3 : 0;
    t.waves_per_block = 1;
    t.chunk_step = -1;
    t.chunk_merge = 8192;
    t.race_probe = -1;
    t.group_r = -1;
    return t;
}

template <int VEC, int OP, bool BF16>
hipError_t launch_nt(const ApplyArgs &a, const ExtArgs *xa, dim3 grid, dim3 bs, hipStream_t st, int nt)
{
    if (xa) {      // extended variants: hints all on or all off
        if (nt & 3) hipLaunchKernelGGL((apply_ext_kernel<VEC, OP, BF16, 3>), grid, bs, 0, st, a, *xa);
        else hipLaunchKernelGGL((apply_ext_kernel<VEC, OP, BF16, 0>), grid, bs, 0, st, a, *xa);
        return hipGetLastError();
    }
    switch (nt & 3) {
    case 0: hipLaunchKernelGGL((apply_kernel<VEC, OP, BF16, 0>), grid, bs, 0, st, a); break;
    case 1: hipLaunchKernelGGL((apply_kernel<VEC, OP, BF16, 1>), grid, bs, 0, st, a); break;
    case 2: hipLaunchKernelGGL((apply_kernel<VEC, OP, BF16, 2>), grid, bs, 0, st, a); break;
    default: hipLaunchKernelGGL((apply_kernel<VEC, OP, BF16, 3>), grid, bs, 0, st, a); break;
    }
    return hipGetLastError();
}

template <int OP, bool BF16>
hipError_t launch_vec(const ApplyArgs &a, const ExtArgs *xa, dim3 grid, dim3 bs, hipStream_t st, int vec, int nt)
{
    switch (vec) {
    case 1: return launch_nt<1, OP, BF16>(a, xa, grid, bs, st, nt);
    case 2: return launch_nt<2, OP, BF16>(a, xa, grid, bs, st, nt);
    default: return launch_nt<4, OP, BF16>(a, xa, grid, bs, st, nt);
    }
}

template <int OP>
hipError_t launch_op(const ApplyArgs &a, const ExtArgs *xa, dim3 grid, dim3 bs, hipStream_t st, int vec, int nt, bool bf16)
{
    return bf16 ? launch_vec<OP, true>(a, xa, grid, bs, st, vec, nt) : launch_vec<OP, false>(a, xa, grid, bs, st, vec, nt);
}

void fill_common(const lasgd_ctx *c, ApplyArgs &a)
{
    a.tiles = c->tiles;
    a.xptr = c->xptr;
    a.gptr = c->gptr;
    a.x32 = c->x32;
    a.v = c->v;
    a.s = c->s;
    a.z = c->z;
    a.npad = c->npad;
    a.ntiles = c->ntiles;
    a.K = (uint32_t)c->K;
    a.n_tensors = (uint32_t)c->n_tensors;
    a.mu = c->mu;
    a.nesterov = c->nesterov;
    a.use_mul = is_pow2((uint32_t)c->K) ? 1 : 0;
    a.inv_k = 1.0 / (double)c->K;
    a.k_as_double = (double)c->K;
}

// A multi-tensor pass, planned (arguments, grid; everything that can be refused)
// and then launched on the main stream.  Callers plan before they enqueue any
// stream dependency, so that a refused call leaves both streams untouched.
struct ApplyPlan {
    ApplyArgs a{};
    int op = 0;
    dim3 grid{1}, bs{64};
    bool has_ext = false;
    ExtArgs ext{};
};

// xa == nullptr: every replica takes part, one step size, alpha = 1 (the plain kernels).
lasgd_status plan_apply(lasgd_ctx *c, ApplyPlan &p, int op, float lr, int resnap, const ExtArgs *xa = nullptr)
{
    if (op < OP_STEP || op > OP_INIT) return fail(c, LASGD_ERR_INVALID, "unknown op %d", op);
    ApplyArgs &a = p.a;
    fill_common(c, a);
    int kper = (op == OP_MERGE || op == OP_STEP_MERGE) ? c->tune.kper_merge : c->tune.kper_step;
    if (kper < 1) kper = 1;
    if (kper > c->K) kper = c->K;
    a.kper = (uint32_t)kper;
    a.kgroups = (uint32_t)((c->K + kper - 1) / kper);
    a.neg_lr = -lr;
    a.resnap = resnap;
    const bool merging = op == OP_MERGE || op == OP_STEP_MERGE;
    int64_t chunk = merging ? c->tune.chunk_merge : c->tune.chunk_step;
    if (chunk < 1 || chunk > (int64_t)a.ntiles) chunk = merging ? 0 : a.ntiles;   // 0: one chunk, handled as the tail
    a.chunk = chunk ? (uint32_t)chunk : 1u;
    const uint32_t nfull = chunk ? a.ntiles / a.chunk : 0u;
    a.full_items = nfull * a.chunk * a.kgroups;
    a.tail_first = nfull * a.chunk;
    const uint32_t tail = a.ntiles - a.tail_first;
    a.tail_chunk = tail ? tail : 1u;
    // passes over the shared z should start on the same XCD for every replica group: 8 XCDs x up to 4 waves
    // per workgroup.  A local step or snapshot reads no z and keeps its items dense.
    a.tail_stride = merging ? (uint32_t)round_up(a.tail_chunk, 32) : a.tail_chunk;
    const uint64_t nitems = (uint64_t)a.full_items + (tail ? (uint64_t)a.tail_stride * a.kgroups : 0u);
    if (nitems == 0 || nitems > 0x7fffffffull) return fail(c, LASGD_ERR_UNSUPPORTED, "work-item count %llu out of range", (unsigned long long)nitems);
    a.nitems = (uint32_t)nitems;
    const uint32_t wpb = (uint32_t)c->tune.waves_per_block;
    uint64_t blocks = (nitems + wpb - 1) / wpb;
    if (c->tune.max_blocks > 0 && blocks > (uint64_t)c->tune.max_blocks) blocks = (uint64_t)c->tune.max_blocks;
    p.op = op;
    p.grid = dim3((uint32_t)blocks);
    p.bs = dim3(64u * wpb);
    p.has_ext = xa != nullptr;
    if (xa) p.ext = *xa;
    return LASGD_OK;
}

lasgd_status launch_apply(lasgd_ctx *c, const ApplyPlan &p)
{
    const bool bf16 = c->storage == LASGD_BF16;
    const int vec = c->tune.vec, nt = c->tune.nontemporal;
    const ExtArgs *xa = p.has_ext ? &p.ext : nullptr;
    hipError_t e = hipSuccess;
    switch (p.op) {
    case OP_STEP: e = launch_op<OP_STEP>(p.a, xa, p.grid, p.bs, c->main, vec, nt, bf16); break;
    case OP_MERGE: e = launch_op<OP_MERGE>(p.a, xa, p.grid, p.bs, c->main, vec, nt, bf16); break;
    case OP_STEP_MERGE: e = launch_op<OP_STEP_MERGE>(p.a, xa, p.grid, p.bs, c->main, vec, nt, bf16); break;
    case OP_SNAPSHOT: e = launch_op<OP_SNAPSHOT>(p.a, xa, p.grid, p.bs, c->main, vec, nt, bf16); break;
    default: e = launch_vec<OP_INIT, true>(p.a, nullptr, p.grid, p.bs, c->main, vec, nt); break;
    }
    if (e != hipSuccess) return fail(c, LASGD_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    return LASGD_OK;
}

lasgd_status enqueue_apply(lasgd_ctx *c, int op, float lr, int resnap, const ExtArgs *xa = nullptr)
{
    ApplyPlan p;
    lasgd_status st = plan_apply(c, p, op, lr, resnap, xa);
    if (st != LASGD_OK) return st;
    return launch_apply(c, p);
}

// The replica-group kernels: one workgroup per tile, W waves, R replicas per wave.
struct GroupShape {
    uint32_t R, W, passes;
    dim3 grid, bs;
    size_t lds;
};

GroupShape group_shape(const lasgd_ctx *c, int kind)
{
    GroupShape g{};
    const uint32_t K = (uint32_t)c->K;
    // replicas a wave takes at a time (measured on MI355X).  Every wave of the SGD-AR kernel
    // repeats the fp64 sum, so it prefers fewer, fatter waves sooner than the fused update,
    // whose sum is shared out; beyond 16 replicas both do best with 8-wave workgroups.
    if (kind == 0) g.R = K < 4u ? 1u : K <= 16u ? 2u : 4u;
    else g.R = K <= kGroupWaves ? 1u : 4u;
    if (c->tune.group_r > 0) g.R = (uint32_t)c->tune.group_r;
    if (g.R > K) g.R = K >= 4 ? 4 : K >= 2 ? 2 : 1;
    g.W = (K + g.R - 1) / g.R;
    if (g.W > kGroupWaves) g.W = kGroupWaves;
    g.passes = (K + g.W * g.R - 1) / (g.W * g.R);
    uint64_t blocks = c->ntiles;
    if (c->tune.max_blocks > 0 && blocks > (uint64_t)c->tune.max_blocks) blocks = (uint64_t)c->tune.max_blocks;
    g.grid = dim3((uint32_t)blocks);
    g.bs = dim3(64u * g.W);
    g.lds = (size_t)K * 256u * sizeof(float);
    return g;
}

template <int KIND, bool BF16, int NT>
hipError_t launch_group_r(const ApplyArgs &a, const GroupShape &g, hipStream_t st)
{
#define LASGD_GROUP(RR)                                                                                  \
    do {                                                                                                 \
        if constexpr (KIND == 0) hipLaunchKernelGGL((sgd_ar_kernel<RR, BF16, NT>), g.grid, g.bs, g.lds, st, a, g.passes); \
        else hipLaunchKernelGGL((step_merge_mean_kernel<RR, BF16, NT>), g.grid, g.bs, g.lds, st, a, g.passes);         \
    } while (0)
    if (g.R == 1) LASGD_GROUP(1);
    else if (g.R == 2) LASGD_GROUP(2);
    else LASGD_GROUP(4);
#undef LASGD_GROUP
    return hipGetLastError();
}

// kind 0: SGD All-Reduce step; kind 1: fused step + global update + next mean
hipError_t launch_group(int kind, const ApplyArgs &a, const GroupShape &g, hipStream_t st, bool bf16, int nt)
{
    const bool hint = (nt & 3) != 0;
    if (kind == 0) {
        if (bf16) return hint ? launch_group_r<0, true, 3>(a, g, st) : launch_group_r<0, true, 0>(a, g, st);
        return hint ? launch_group_r<0, false, 3>(a, g, st) : launch_group_r<0, false, 0>(a, g, st);
    }
    if (bf16) return hint ? launch_group_r<1, true, 3>(a, g, st) : launch_group_r<1, true, 0>(a, g, st);
    return hint ? launch_group_r<1, false, 3>(a, g, st) : launch_group_r<1, false, 0>(a, g, st);
}

template <bool EXT>
hipError_t launch_average(const AvgArgs &a, dim3 grid, hipStream_t st, int split, bool nt, uint32_t bs1)
{
    if (split == 1) {
        if (nt) hipLaunchKernelGGL((average_kernel<3, EXT>), grid, dim3(bs1), 0, st, a);
        else hipLaunchKernelGGL((average_kernel<0, EXT>), grid, dim3(bs1), 0, st, a);
    } else if (split == 2) {
        if (nt) hipLaunchKernelGGL((average_split_kernel<2, 3, EXT>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((average_split_kernel<2, 0, EXT>), grid, dim3(256), 0, st, a);
    } else {
        if (nt) hipLaunchKernelGGL((average_split_kernel<4, 3, EXT>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((average_split_kernel<4, 0, EXT>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

// Enqueue the mean of the replicas in `mask` on the side stream.
lasgd_status enqueue_average(lasgd_ctx *c, uint64_t mask, bool elastic)
{
    AvgArgs a{};
    a.s = c->s;
    a.z = c->z;
    a.npad = c->npad;
    a.nvec = c->npad / 4;
    uint32_t kp = 0;
    for (int k = 0; k < c->K; ++k)
        if ((mask >> k) & 1ull) a.idx[kp++] = (uint8_t)k;
    a.K = kp;
    a.use_mul = is_pow2(kp) ? 1 : 0;
    a.inv_k = 1.0 / (double)kp;
    a.k_as_double = (double)kp;
    a.elastic = elastic ? 1 : 0;
    a.beta = (double)c->beta;
    a.one_minus_beta = 1.0 - (double)c->beta;
    const int split = c->tune.avg_split;
    const uint32_t bs1 = 64u * (uint32_t)c->tune.waves_per_block;           // block size of the unsplit kernel
    const uint64_t cols = split == 1 ? bs1 : 256u / (uint32_t)split;
    uint64_t blocks = (a.nvec + cols - 1) / cols;
    if (c->tune.avg_max_blocks > 0 && blocks > (uint64_t)c->tune.avg_max_blocks) blocks = (uint64_t)c->tune.avg_max_blocks;
    if (blocks > 0x7fffffffull) blocks = 0x7fffffffull;
    const dim3 grid((uint32_t)blocks);
    const bool nt = (c->tune.nontemporal & 1) != 0;
    const bool ext = elastic || mask != c->all;
    hipError_t e = ext ? launch_average<true>(a, grid, c->side, split, nt, bs1) : launch_average<false>(a, grid, c->side, split, nt, bs1);
    if (e != hipSuccess) return fail(c, LASGD_ERR_HIP, "average launch failed: %s", hipGetErrorString(e));
    return LASGD_OK;
}

lasgd_status check_ready_to_step(lasgd_ctx *c, float lr)
{
    if (!std::isfinite(lr)) return fail(c, LASGD_ERR_INVALID, "learning rate is not finite");
    if (c->n_bound != c->K) return fail(c, LASGD_ERR_STATE, "%d of %d replicas are bound", c->n_bound, c->K);
    if (c->storage == LASGD_BF16 && !c->master_ready)
        return fail(c, LASGD_ERR_STATE, "bf16 storage: call lasgd_init_master first");
    return LASGD_OK;
}

void release(lasgd_ctx *c)
{
    if (c->arena) (void)hipFree(c->arena);
    for (Tile *t : c->tiles_by_vec)
        if (t) (void)hipFree(t);
    if (c->xptr) (void)hipFree(c->xptr);
    if (c->evA) (void)hipEventDestroy(c->evA);
    if (c->evZ) (void)hipEventDestroy(c->evZ);
    delete c;
}

} // namespace

static lasgd_status create_impl(const lasgd_config *cfg, lasgd_ctx **out)
{
    if (out) *out = nullptr;
    if (!cfg || !out) return fail(nullptr, LASGD_ERR_INVALID, "NULL argument");
    if (cfg->K < 1 || cfg->K > kMaxK) return fail(nullptr, LASGD_ERR_INVALID, "K = %d outside 1..%d", cfg->K, kMaxK);
    if (cfg->n_tensors < 1 || !cfg->numel) return fail(nullptr, LASGD_ERR_INVALID, "empty parameter list");
    if (cfg->storage != LASGD_F32 && cfg->storage != LASGD_BF16) return fail(nullptr, LASGD_ERR_INVALID, "unknown storage dtype");
    if (!std::isfinite(cfg->momentum) || cfg->momentum < 0.f) return fail(nullptr, LASGD_ERR_INVALID, "momentum must be finite and >= 0");
    if (!std::isfinite(cfg->wd_scalar) || cfg->wd_scalar < 0.f) return fail(nullptr, LASGD_ERR_INVALID, "weight decay must be finite and >= 0");
    lasgd_ctx *c = new (std::nothrow) lasgd_ctx;
    if (!c) return fail(nullptr, LASGD_ERR_ALLOC, "out of host memory");
    c->K = cfg->K;
    c->n_tensors = cfg->n_tensors;
    c->storage = cfg->storage;
    c->mu = cfg->momentum;
    c->nesterov = cfg->nesterov ? 1 : 0;
    c->wd_scalar = cfg->wd_scalar;
    c->main = (hipStream_t)cfg->main_stream;
    c->side = (hipStream_t)cfg->side_stream;
    uint64_t off = 0, total = 0;
    for (int32_t i = 0; i < cfg->n_tensors; ++i) {
        if (cfg->numel[i] < 1) { delete c; return fail(nullptr, LASGD_ERR_INVALID, "numel[%d] = %lld", i, (long long)cfg->numel[i]); }
        const float w = cfg->weight_decay ? cfg->weight_decay[i] : cfg->wd_scalar;
        if (!std::isfinite(w) || w < 0.f) { delete c; return fail(nullptr, LASGD_ERR_INVALID, "weight_decay[%d] must be finite and >= 0", i); }
        c->numel.push_back(cfg->numel[i]);
        c->wd.push_back(w);
        c->aoff.push_back(off);
        total += (uint64_t)cfg->numel[i];
        off += round_up((uint64_t)cfg->numel[i], kArenaAlign);
        if (off > kMaxNpad) { delete c; return fail(nullptr, LASGD_ERR_UNSUPPORTED, "more than %llu elements per replica", (unsigned long long)kMaxNpad); }
    }
    c->npad = off;
    c->all = c->K == 64 ? ~0ull : ((1ull << c->K) - 1ull);
    c->ntotal = total;
    c->bound.assign((size_t)c->K, 0);
    c->h_xptr.assign((size_t)c->K * c->n_tensors, nullptr);
    c->h_gptr.assign((size_t)c->K * c->n_tensors, nullptr);
    c->tune = default_tuning(*c);

#define CREATE_HIP(call)                                                                       \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess) {                                                                \
            (void)hipGetLastError();                                                           \
            lasgd_status st_ = fail(nullptr, e_ == hipErrorOutOfMemory ? LASGD_ERR_ALLOC : LASGD_ERR_HIP, \
                                    "%s failed: %s", #call, hipGetErrorString(e_));            \
            release(c);                                                                        \
            return st_;                                                                        \
        }                                                                                      \
    } while (0)

    CREATE_HIP(hipGetDevice(&c->device));
    const bool bf16 = c->storage == LASGD_BF16;
    const uint64_t per = c->npad * sizeof(float);
    const uint64_t n_arrays = (uint64_t)c->K * (bf16 ? 3 : 2) + 1;       // v, s (, x32), z
    CREATE_HIP(hipMalloc((void **)&c->arena, n_arrays * per));
    CREATE_HIP(hipMemsetAsync(c->arena, 0, n_arrays * per, c->main));
    c->v = (float *)c->arena;
    c->s = c->v + (uint64_t)c->K * c->npad;
    c->z = c->s + (uint64_t)c->K * c->npad;
    c->x32 = bf16 ? c->z + c->npad : nullptr;
    const size_t tab = (size_t)c->K * c->n_tensors * sizeof(void *);
    CREATE_HIP(hipMalloc((void **)&c->xptr, 2 * tab));
    c->gptr = c->xptr + (size_t)c->K * c->n_tensors;
    CREATE_HIP(hipMemset(c->xptr, 0, 2 * tab));
    CREATE_HIP(hipEventCreateWithFlags(&c->evA, hipEventDisableTiming));
    CREATE_HIP(hipEventCreateWithFlags(&c->evZ, hipEventDisableTiming));
    lasgd_status st = upload_tiles(c, c->tune.vec);
    if (st != LASGD_OK) {
        g_create_error = c->err;
        release(c);
        return st;
    }
    CREATE_HIP(hipStreamSynchronize(c->main));
#undef CREATE_HIP
    *out = c;
    return LASGD_OK;
}

extern "C" {

// Host containers may throw on exhaustion; nothing may leave through the C ABI.
lasgd_status lasgd_create(const lasgd_config *cfg, lasgd_ctx **out)
{
    try {
        return create_impl(cfg, out);
    } catch (...) {
        if (out) *out = nullptr;
        try { g_create_error = "out of host memory"; } catch (...) {}
        return LASGD_ERR_ALLOC;
    }
}

lasgd_status lasgd_bind(lasgd_ctx *c, int32_t k, void *const *params, void *const *grads)
{
    if (!c) return LASGD_ERR_INVALID;
    if (!params || !grads) return fail(c, LASGD_ERR_INVALID, "NULL pointer array");
    if (k < 0 || k >= c->K) return fail(c, LASGD_ERR_INVALID, "replica %d outside 0..%d", k, c->K - 1);
    for (int32_t t = 0; t < c->n_tensors; ++t) {
        if (!params[t] || !grads[t]) return fail(c, LASGD_ERR_INVALID, "NULL buffer for tensor %d", t);
        if (((uintptr_t)params[t] | (uintptr_t)grads[t]) & 15u)
            return fail(c, LASGD_ERR_INVALID, "buffer of tensor %d is not 16-byte aligned", t);
    }
    LASGD_HIP(c, hipStreamSynchronize(c->main));
    const size_t base = (size_t)k * c->n_tensors, bytes = (size_t)c->n_tensors * sizeof(void *);
    LASGD_HIP(c, hipMemcpy(c->xptr + base, params, bytes, hipMemcpyHostToDevice));
    LASGD_HIP(c, hipMemcpy(c->gptr + base, grads, bytes, hipMemcpyHostToDevice));
    memcpy(&c->h_xptr[base], params, bytes);
    memcpy(&c->h_gptr[base], grads, bytes);
    if (!c->bound[(size_t)k]) {
        c->bound[(size_t)k] = 1;
        ++c->n_bound;
    }
    return LASGD_OK;
}

lasgd_status lasgd_init_master(lasgd_ctx *c)
{
    if (!c) return LASGD_ERR_INVALID;
    if (c->storage != LASGD_BF16) return fail(c, LASGD_ERR_STATE, "storage is fp32: there is no master copy");
    if (c->n_bound != c->K) return fail(c, LASGD_ERR_STATE, "%d of %d replicas are bound", c->n_bound, c->K);
    if (c->pending_mask) return fail(c, LASGD_ERR_STATE, "an average is in flight");
    lasgd_status st = enqueue_apply(c, OP_INIT, 0.f, 0);
    if (st != LASGD_OK) return st;
    c->master_ready = true;
    c->snap_mask = 0;
    return LASGD_OK;
}

// ---- shared by the plain and the extended entry points -------------------
// The plain calls are the extended ones with every replica taking part, one
// step size and alpha = 1; they launch the lean kernels.

static lasgd_status check_mask(lasgd_ctx *c, uint64_t mask, bool may_be_empty, const char *what)
{
    if (mask & ~c->all) return fail(c, LASGD_ERR_INVALID, "%s names replicas beyond K = %d", what, c->K);
    if (!may_be_empty && !mask) return fail(c, LASGD_ERR_INVALID, "%s is empty", what);
    return LASGD_OK;
}

static lasgd_status check_lrs(lasgd_ctx *c, const float *lr, uint64_t mask)
{
    if (!lr) return fail(c, LASGD_ERR_INVALID, "NULL learning-rate array");
    for (int k = 0; k < c->K; ++k)
        if (((mask >> k) & 1ull) && !std::isfinite(lr[k])) return fail(c, LASGD_ERR_INVALID, "learning rate of replica %d is not finite", k);
    return LASGD_OK;
}

static bool fill_ext(const lasgd_ctx *c, ExtArgs &x, const float *lr, uint64_t step_mask, uint64_t merge_mask)
{
    x.step_mask = step_mask;
    x.merge_mask = merge_mask;
    x.alpha = c->alpha;
    bool uniform = true;
    float first = 0.f;
    bool have = false;
    for (int k = 0; k < 64; ++k) {
        const bool in = k < c->K && ((step_mask >> k) & 1ull) && lr;
        x.neg_lr_k[k] = in ? -lr[k] : 0.f;
        if (in) {
            if (!have) { first = lr[k]; have = true; }
            else if (lr[k] != first) uniform = false;
        }
    }
    return uniform;
}

static lasgd_status do_local_step(lasgd_ctx *c, const float *lr_k, float lr, uint64_t mask)
{
    lasgd_status st = check_ready_to_step(c, lr_k ? 0.f : lr);
    if (st != LASGD_OK) return st;
    if (!lr_k && mask == c->all) return enqueue_apply(c, OP_STEP, lr, 0);
    if ((st = check_mask(c, mask, true, "mask")) != LASGD_OK) return st;
    if ((st = check_lrs(c, lr_k, mask)) != LASGD_OK) return st;
    if (!mask) return LASGD_OK;                        // nobody steps: nothing to enqueue
    ExtArgs x{};
    const bool uniform = fill_ext(c, x, lr_k, mask, 0);
    if (uniform && mask == c->all) return enqueue_apply(c, OP_STEP, lr_k[0], 0);
    return enqueue_apply(c, OP_STEP, 0.f, 0, &x);
}

static lasgd_status do_snapshot(lasgd_ctx *c, uint64_t mask)
{
    lasgd_status st = check_ready_to_step(c, 0.f);
    if (st != LASGD_OK) return st;
    if ((st = check_mask(c, mask, false, "mask")) != LASGD_OK) return st;
    if (mask & c->pending_mask)
        return fail(c, LASGD_ERR_STATE, "an average over some of these replicas is in flight and not merged: s may still be read");
    if (mask == c->all) st = enqueue_apply(c, OP_SNAPSHOT, 0.f, 0);
    else {
        ExtArgs x{};
        fill_ext(c, x, nullptr, mask, 0);
        st = enqueue_apply(c, OP_SNAPSHOT, 0.f, 0, &x);
    }
    if (st != LASGD_OK) return st;
    c->snap_mask |= mask;
    return LASGD_OK;
}

// Is this stream recording into a graph rather than executing?
static bool is_capturing(hipStream_t st)
{
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return cs != hipStreamCaptureStatusNone;
}

static lasgd_status do_average(lasgd_ctx *c, uint64_t mask)
{
    // every refusal comes before the first event or launch
    lasgd_status st = check_mask(c, mask, false, "mask");
    if (st != LASGD_OK) return st;
    if (c->pending_mask) return fail(c, LASGD_ERR_STATE, "the previous average has not been merged by all its participants");
    if (mask & ~c->snap_mask) return fail(c, LASGD_ERR_STATE, "no snapshot to average for some of these replicas");
    const bool captured = is_capturing(c->main);
    if (c->side != c->main) {
        LASGD_HIP(c, hipEventRecord(c->evA, c->main));
        LASGD_HIP(c, hipStreamWaitEvent(c->side, c->evA, 0));
    }
    // the first mean initialises the centre: there is no earlier z to blend with
    const bool elastic = c->beta != 1.f && c->center_valid;
    if (c->tune.race_probe > 0 && !elastic) {
        // debugging aid: z is poisoned on the side stream just before the mean rewrites it
        hipLaunchKernelGGL(poison_kernel, dim3(1024), dim3(256), 0, c->side, c->z, c->npad);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(c, LASGD_ERR_HIP, "poison launch failed: %s", hipGetErrorString(e));
    }
    st = enqueue_average(c, mask, elastic);
    if (st != LASGD_OK) return st;
    // from here on the side stream reads s and writes z: the state says so even if the event below fails
    c->pending_mask = mask;
    c->avg_ever = true;
    c->center_valid = true;
    c->avg_in_graph = captured;
    c->z_on_main = c->side == c->main;
    LASGD_HIP(c, hipEventRecord(c->evZ, c->side));
    return LASGD_OK;
}

static lasgd_status do_merge(lasgd_ctx *c, int op, const float *lr_k, float lr, uint64_t step_mask,
                             uint64_t merge_mask, int32_t resnapshot)
{
    lasgd_status st = check_ready_to_step(c, lr_k ? 0.f : lr);
    if (st != LASGD_OK) return st;
    if ((st = check_mask(c, merge_mask, false, "merge mask")) != LASGD_OK) return st;
    if ((st = check_mask(c, step_mask, true, "step mask")) != LASGD_OK) return st;
    if (op == OP_STEP_MERGE && lr_k && (st = check_lrs(c, lr_k, step_mask)) != LASGD_OK) return st;
    if (!c->pending_mask) return fail(c, LASGD_ERR_STATE, "no average launched since the last merge");
    if (merge_mask & ~c->pending_mask)
        return fail(c, LASGD_ERR_STATE, "some of these replicas did not take part in the pending average or have merged already");
    ExtArgs x{};
    float same[64];
    for (int k = 0; k < 64; ++k) same[k] = lr;
    const bool uniform = fill_ext(c, x, lr_k ? lr_k : same, step_mask, merge_mask);
    const bool plain = merge_mask == c->all && c->alpha == 1.f &&
                       (op == OP_MERGE || (step_mask == c->all && uniform));
    ApplyPlan p;
    if (plain) st = plan_apply(c, p, op, lr_k ? lr_k[0] : lr, resnapshot ? 1 : 0);
    else st = plan_apply(c, p, op, 0.f, resnapshot ? 1 : 0, &x);
    if (st != LASGD_OK) return st;
    // nothing can be refused any more: now the main stream waits for z (unless z is made on this very stream)
    if (!c->z_on_main) LASGD_HIP(c, hipStreamWaitEvent(c->main, c->evZ, 0));
    st = launch_apply(c, p);
    if (st != LASGD_OK) return st;
    c->pending_mask &= ~merge_mask;
    if (resnapshot) c->snap_mask |= merge_mask;
    else c->snap_mask &= ~merge_mask;
    return LASGD_OK;
}

lasgd_status lasgd_local_step(lasgd_ctx *c, float lr)
{
    if (!c) return LASGD_ERR_INVALID;
    return do_local_step(c, nullptr, lr, c->all);
}

lasgd_status lasgd_local_step_ex(lasgd_ctx *c, const float *lr, uint64_t mask)
{
    if (!c) return LASGD_ERR_INVALID;
    if (!lr) return fail(c, LASGD_ERR_INVALID, "NULL learning-rate array");
    return do_local_step(c, lr, 0.f, mask);
}

lasgd_status lasgd_snapshot(lasgd_ctx *c)
{
    if (!c) return LASGD_ERR_INVALID;
    return do_snapshot(c, c->all);
}

lasgd_status lasgd_snapshot_ex(lasgd_ctx *c, uint64_t mask)
{
    if (!c) return LASGD_ERR_INVALID;
    return do_snapshot(c, mask);
}

lasgd_status lasgd_average(lasgd_ctx *c)
{
    if (!c) return LASGD_ERR_INVALID;
    return do_average(c, c->all);
}

lasgd_status lasgd_average_ex(lasgd_ctx *c, uint64_t mask)
{
    if (!c) return LASGD_ERR_INVALID;
    return do_average(c, mask);
}

lasgd_status lasgd_average_done(lasgd_ctx *c, int32_t *done)
{
    if (!c) return LASGD_ERR_INVALID;
    if (!done) return fail(c, LASGD_ERR_INVALID, "NULL argument");
    if (!c->avg_ever) return fail(c, LASGD_ERR_STATE, "no average has been launched");
    if (c->avg_in_graph)
        return fail(c, LASGD_ERR_STATE, "the last average was recorded into a graph: its completion cannot be polled here");
    hipError_t e = hipEventQuery(c->evZ);
    if (e == hipSuccess) *done = 1;
    else if (e == hipErrorNotReady) *done = 0;
    else return fail(c, LASGD_ERR_HIP, "hipEventQuery failed: %s", hipGetErrorString(e));
    return LASGD_OK;
}

lasgd_status lasgd_merge(lasgd_ctx *c, int32_t resnapshot)
{
    if (!c) return LASGD_ERR_INVALID;
    return do_merge(c, OP_MERGE, nullptr, 0.f, 0, c->all, resnapshot);
}

lasgd_status lasgd_merge_ex(lasgd_ctx *c, uint64_t mask, int32_t resnapshot)
{
    if (!c) return LASGD_ERR_INVALID;
    return do_merge(c, OP_MERGE, nullptr, 0.f, 0, mask, resnapshot);
}

lasgd_status lasgd_step_merge(lasgd_ctx *c, float lr, int32_t resnapshot)
{
    if (!c) return LASGD_ERR_INVALID;
    return do_merge(c, OP_STEP_MERGE, nullptr, lr, c->all, c->all, resnapshot);
}

lasgd_status lasgd_step_merge_ex(lasgd_ctx *c, const float *lr, uint64_t step_mask, uint64_t merge_mask,
                                 int32_t resnapshot)
{
    if (!c) return LASGD_ERR_INVALID;
    if (!lr) return fail(c, LASGD_ERR_INVALID, "NULL learning-rate array");
    return do_merge(c, OP_STEP_MERGE, lr, 0.f, step_mask, merge_mask, resnapshot);
}

lasgd_status lasgd_set_elastic(lasgd_ctx *c, float alpha, float beta)
{
    if (!c) return LASGD_ERR_INVALID;
    if (!(alpha >= 0.f && alpha <= 1.f) || !(beta >= 0.f && beta <= 1.f))
        return fail(c, LASGD_ERR_INVALID, "alpha and beta must lie in [0, 1]");
    c->alpha = alpha;
    c->beta = beta;
    return LASGD_OK;
}

lasgd_status lasgd_sgd_ar_step(lasgd_ctx *c, float lr)
{
    if (!c) return LASGD_ERR_INVALID;
    lasgd_status st = check_ready_to_step(c, lr);
    if (st != LASGD_OK) return st;
    ApplyArgs a{};
    fill_common(c, a);
    a.neg_lr = -lr;
    const GroupShape g = group_shape(c, 0);
    hipError_t e = launch_group(0, a, g, c->main, c->storage == LASGD_BF16, c->tune.nontemporal);
    if (e != hipSuccess) return fail(c, LASGD_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    return LASGD_OK;
}

lasgd_status lasgd_step_merge_average(lasgd_ctx *c, float lr)
{
    if (!c) return LASGD_ERR_INVALID;
    lasgd_status st = check_ready_to_step(c, lr);
    if (st != LASGD_OK) return st;
    if (!c->pending_mask) return fail(c, LASGD_ERR_STATE, "no average launched since the last merge");
    if (c->pending_mask != c->all)
        return fail(c, LASGD_ERR_STATE, "the pending average is partial or partly merged: use lasgd_step_merge_ex and lasgd_average_ex");
    if (c->alpha != 1.f || c->beta != 1.f)
        return fail(c, LASGD_ERR_STATE, "elastic coefficients are set: use lasgd_step_merge and lasgd_average");
    ApplyArgs a{};
    fill_common(c, a);
    a.neg_lr = -lr;
    a.resnap = 1;
    const GroupShape g = group_shape(c, 1);
    const bool captured = is_capturing(c->main);
    if (!c->z_on_main) LASGD_HIP(c, hipStreamWaitEvent(c->main, c->evZ, 0));
    hipError_t e = launch_group(1, a, g, c->main, c->storage == LASGD_BF16, c->tune.nontemporal);
    if (e != hipSuccess) return fail(c, LASGD_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    // every replica has merged and re-sent, and the mean of the sent models is (being) written to z
    // on the main stream: the same state as after lasgd_step_merge(lr, 1) + lasgd_average
    c->snap_mask = c->all;
    c->pending_mask = c->all;
    c->avg_in_graph = captured;
    c->z_on_main = true;
    LASGD_HIP(c, hipEventRecord(c->evZ, c->main));
    return LASGD_OK;
}

lasgd_status lasgd_sync(lasgd_ctx *c)
{
    if (!c) return LASGD_ERR_INVALID;
    LASGD_HIP(c, hipStreamSynchronize(c->main));
    if (c->side != c->main) LASGD_HIP(c, hipStreamSynchronize(c->side));
    return LASGD_OK;
}

lasgd_status lasgd_read_state(lasgd_ctx *c, int32_t which, int32_t k, int32_t tensor, float *dst, int64_t n)
{
    if (!c) return LASGD_ERR_INVALID;
    if (!dst) return fail(c, LASGD_ERR_INVALID, "NULL destination");
    if (which < LASGD_STATE_X || which > LASGD_STATE_Z) return fail(c, LASGD_ERR_INVALID, "unknown state array %d", which);
    if (which == LASGD_STATE_Z) k = 0;
    if (k < 0 || k >= c->K) return fail(c, LASGD_ERR_INVALID, "replica %d outside 0..%d", k, c->K - 1);
    if (tensor < -1 || tensor >= c->n_tensors) return fail(c, LASGD_ERR_INVALID, "tensor %d outside -1..%d", tensor, c->n_tensors - 1);
    const int64_t want = tensor < 0 ? (int64_t)c->ntotal : c->numel[(size_t)tensor];
    if (n != want) return fail(c, LASGD_ERR_INVALID, "n = %lld, expected %lld", (long long)n, (long long)want);
    const bool user_x = which == LASGD_STATE_X && c->storage == LASGD_F32;
    if (user_x && !c->bound[(size_t)k]) return fail(c, LASGD_ERR_STATE, "replica %d is not bound", k);
    lasgd_status st = lasgd_sync(c);
    if (st != LASGD_OK) return st;
    const float *base = which == LASGD_STATE_V ? c->v : which == LASGD_STATE_S ? c->s : which == LASGD_STATE_Z ? c->z : c->x32;
    const int32_t t0 = tensor < 0 ? 0 : tensor, t1 = tensor < 0 ? c->n_tensors : tensor + 1;
    float *out = dst;
    for (int32_t t = t0; t < t1; ++t) {
        const void *src = user_x ? c->h_xptr[(size_t)k * c->n_tensors + t]
                                 : (const void *)(base + (which == LASGD_STATE_Z ? 0 : (uint64_t)k * c->npad) + c->aoff[(size_t)t]);
        LASGD_HIP(c, hipMemcpy(out, src, (size_t)c->numel[(size_t)t] * sizeof(float), hipMemcpyDeviceToHost));
        out += c->numel[(size_t)t];
    }
    return LASGD_OK;
}

static lasgd_status set_tuning_impl(lasgd_ctx *c, const lasgd_tuning *t)
{
    if (!c) return LASGD_ERR_INVALID;
    if (!t) return fail(c, LASGD_ERR_INVALID, "NULL argument");
    lasgd_tuning n = c->tune;
    if (t->vec) {
        if (t->vec != 1 && t->vec != 2 && t->vec != 4) return fail(c, LASGD_ERR_INVALID, "vec must be 1, 2 or 4");
        n.vec = t->vec;
    }
    if (t->kper_step) {
        if (t->kper_step < 1 || t->kper_step > c->K) return fail(c, LASGD_ERR_INVALID, "kper_step outside 1..K");
        n.kper_step = t->kper_step;
    }
    if (t->kper_merge) {
        if (t->kper_merge < 1 || t->kper_merge > c->K) return fail(c, LASGD_ERR_INVALID, "kper_merge outside 1..K");
        n.kper_merge = t->kper_merge;
    }
    if (t->max_blocks) n.max_blocks = t->max_blocks;
    if (t->avg_split) {
        if (t->avg_split != 1 && t->avg_split != 2 && t->avg_split != 4) return fail(c, LASGD_ERR_INVALID, "avg_split must be 1, 2 or 4");
        n.avg_split = t->avg_split;
    }
    if (t->avg_max_blocks) n.avg_max_blocks = t->avg_max_blocks;
    if (t->nontemporal) {
        if (t->nontemporal < 0 || t->nontemporal > 4) return fail(c, LASGD_ERR_INVALID, "nontemporal outside 0..4");
        n.nontemporal = t->nontemporal == 4 ? 0 : t->nontemporal;      // 4 = switch the hints off again
    }
    if (t->waves_per_block) {
        if (t->waves_per_block != 1 && t->waves_per_block != 2 && t->waves_per_block != 4)
            return fail(c, LASGD_ERR_INVALID, "waves_per_block must be 1, 2 or 4");
        n.waves_per_block = t->waves_per_block;
    }
    if (t->chunk_step) n.chunk_step = t->chunk_step < 0 ? -1 : t->chunk_step;
    if (t->chunk_merge) n.chunk_merge = t->chunk_merge < 0 ? -1 : t->chunk_merge;
    if (t->race_probe) n.race_probe = t->race_probe > 0 ? 1 : -1;
    if (t->group_r) {
        if (t->group_r > 0 && t->group_r != 1 && t->group_r != 2 && t->group_r != 4)
            return fail(c, LASGD_ERR_INVALID, "group_r must be 1, 2 or 4 (or negative for the default)");
        n.group_r = t->group_r < 0 ? -1 : t->group_r;
    }
    lasgd_status st = lasgd_sync(c);
    if (st != LASGD_OK) return st;
    if (n.vec != c->tune.vec) {
        st = upload_tiles(c, n.vec);
        if (st != LASGD_OK) return st;
    }
    c->tune = n;
    return LASGD_OK;
}

lasgd_status lasgd_set_tuning(lasgd_ctx *c, const lasgd_tuning *t)
{
    try {
        return set_tuning_impl(c, t);
    } catch (...) {
        return LASGD_ERR_ALLOC;
    }
}

lasgd_status lasgd_get_tuning(const lasgd_ctx *c, lasgd_tuning *out)
{
    if (!c || !out) return LASGD_ERR_INVALID;
    *out = c->tune;
    return LASGD_OK;
}

const char *lasgd_last_error(const lasgd_ctx *c)
{
    return c ? c->err.c_str() : g_create_error.c_str();
}

void lasgd_destroy(lasgd_ctx *c)
{
    if (!c) return;
    (void)hipStreamSynchronize(c->main);
    if (c->side != c->main) (void)hipStreamSynchronize(c->side);
    release(c);
}

} // extern "C"

// ---- the allocation-free entry point ---------------------------------------
// z of lasgd_global_update_static lives in this file-scope device array instead
// of an allocation.  Every GPU that loads the library holds its own copy (128 MiB)
// until the process ends.  In host code the array's name is only a stand-in for
// the symbol; its device address is looked up once per device and that pointer
// is what kernels and copies receive.
constexpr int64_t kStaticMaxN = LASGD_STATIC_MAX_N;
static __device__ __align__(256) float scratch[kStaticMaxN];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on first use).
lasgd_status scratch_for_current_device(float **out)
{
    int dev = -1;
    LASGD_HIP(nullptr, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, LASGD_ERR_UNSUPPORTED, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        float *p = nullptr;
        LASGD_HIP(nullptr, hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(nullptr, LASGD_ERR_HIP, "hipGetSymbolAddress returned a NULL address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LASGD_OK;
}

} // namespace

extern "C" lasgd_status lasgd_global_update_static(int32_t K, int64_t n, float *const *x, float *const *sent,
                                                   int32_t resnapshot, void *stream)
{
    try {
        if (!x || !sent) return fail(nullptr, LASGD_ERR_INVALID, "NULL pointer array");
        if (K < 1 || K > kMaxK) return fail(nullptr, LASGD_ERR_INVALID, "K = %d outside 1..%d", K, kMaxK);
        if (n < 1) return fail(nullptr, LASGD_ERR_INVALID, "n = %lld: nothing to update", (long long)n);
        if (n > kStaticMaxN)
            return fail(nullptr, LASGD_ERR_UNSUPPORTED,
                        "n = %lld exceeds the static buffer of this entry point (LASGD_STATIC_MAX_N = %lld elements); "
                        "split the vector or use a context",
                        (long long)n, (long long)kStaticMaxN);
        FlatArgs a{};
        for (int32_t k = 0; k < K; ++k) {
            if (!x[k] || !sent[k]) return fail(nullptr, LASGD_ERR_INVALID, "NULL buffer for replica %d", k);
            if (((uintptr_t)x[k] | (uintptr_t)sent[k]) & 15u)
                return fail(nullptr, LASGD_ERR_INVALID, "buffer of replica %d is not 16-byte aligned", k);
            a.x[k] = x[k];
            a.s[k] = sent[k];
        }
        // the 2K buffers must not overlap: every one of them is written by one replica's waves only
        const uintptr_t bytes = (uintptr_t)n * sizeof(float);
        for (int32_t i = 0; i < 2 * K; ++i)
            for (int32_t j = 0; j < i; ++j) {
                const uintptr_t p = (uintptr_t)(i < K ? x[i] : sent[i - K]), q = (uintptr_t)(j < K ? x[j] : sent[j - K]);
                if (p < q + bytes && q < p + bytes)
                    return fail(nullptr, LASGD_ERR_INVALID, "%s of replica %d overlaps %s of replica %d",
                                i < K ? "x" : "sent", i < K ? i : i - K, j < K ? "x" : "sent", j < K ? j : j - K);
            }
        float *z = nullptr;
        lasgd_status st = scratch_for_current_device(&z);
        if (st != LASGD_OK) return st;
        a.z = z;
        a.n = (uint64_t)n;
        a.nvec = (uint64_t)n / 4u;
        a.K = (uint32_t)K;
        a.use_mul = is_pow2((uint32_t)K) ? 1 : 0;
        a.inv_k = 1.0 / (double)K;
        a.k_as_double = (double)K;
        a.resnap = resnapshot ? 1 : 0;
        hipStream_t hs = (hipStream_t)stream;
        // one thread per 128-bit vector, at least enough threads for the scalar tail
        uint64_t blocks = (a.nvec + 255u) / 256u;
        if (blocks < 1) blocks = 1;
        if (blocks > 65535u * 16u) blocks = 65535u * 16u;
        hipLaunchKernelGGL(flat_mean_kernel, dim3((uint32_t)blocks), dim3(256), 0, hs, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(nullptr, LASGD_ERR_HIP, "mean launch failed: %s", hipGetErrorString(e));
        hipLaunchKernelGGL(flat_merge_kernel, dim3((uint32_t)blocks, (uint32_t)K), dim3(256), 0, hs, a);
        e = hipGetLastError();
        if (e != hipSuccess) return fail(nullptr, LASGD_ERR_HIP, "global-update launch failed: %s", hipGetErrorString(e));
        return LASGD_OK;
    } catch (...) {
        return LASGD_ERR_ALLOC;
    }
}
