// Device half of the library: index upload, workspace planning, kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <functional>
#include <mutex>

#include "etf_internal.h"
#include "etf_kernels.hip.h"
#include "etf_ctx_kernels.hip.h"

using namespace etf;

#define HIP_TRY(ctx, call)                                                                            \
    do {                                                                                              \
        hipError_t e_ = (call);                                                                       \
        if (e_ != hipSuccess) return fail(ctx, ETF_EHIP, "%s: %s", #call, hipGetErrorString(e_));     \
    } while (0)

#define LAUNCH_CHECK(ctx, name)                                                                       \
    do {                                                                                              \
        hipError_t e_ = hipGetLastError();                                                            \
        if (e_ != hipSuccess) return fail(ctx, ETF_EHIP, "launch of %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

// Brackets the launches made during its lifetime with a pair of events when profiling is on.
struct ProfScope {
    etf_ctx *ctx;
    etf_ctx::Stamp st{nullptr, nullptr, 0};
    bool live = false;
    ProfScope(etf_ctx *c, int cls) : ctx(c)
    {
        if (!c->profile_on || c->no_alloc_call) return;
        if (!c->stamp_pool.empty()) {
            st = c->stamp_pool.back();
            c->stamp_pool.pop_back();
        } else {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess) return;
            if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
            st.start = a;
            st.stop = b;
        }
        st.cls = cls;
        live = hipEventRecord((hipEvent_t)st.start, (hipStream_t)c->stream) == hipSuccess;
        if (!live) c->stamp_pool.push_back(st);
    }
    ~ProfScope()
    {
        if (!live) return;
        (void)hipEventRecord((hipEvent_t)st.stop, (hipStream_t)ctx->stream);
        ctx->stamps.push_back(st);
    }
};

static void lookup_scratch(int device);

static constexpr int64_t LDS_BUDGET = 128 * 1024;  // bytes of table slices a workgroup may stage
static constexpr int CUB = 4;                       // items per batch of the register-context kernels (measured best)

// =============================================================================================
// context
// =============================================================================================
extern "C" int etf_create(etf_ctx **out, int device, void *hip_stream)
{
    if (!out) return ETF_EINVAL;
    *out = nullptr;
    if (device >= 0) {
        int n = 0;
        if (hipGetDeviceCount(&n) != hipSuccess || device >= n) return ETF_ENOGPU;
    }
    etf_ctx *c = new (std::nothrow) etf_ctx();
    if (!c) return ETF_ENOMEM;
    c->device = device;
    c->stream = hip_stream;
    if (device >= 0) lookup_scratch(device);  // once per device: where the scratch of etf_search_static lives there
    *out = c;
    return ETF_OK;
}

extern "C" void etf_destroy(etf_ctx *ctx)
{
    if (!ctx) return;
    for (auto *v : {&ctx->stamps, &ctx->stamp_pool})
        for (auto &s : *v) {
            (void)hipEventDestroy((hipEvent_t)s.start);
            (void)hipEventDestroy((hipEvent_t)s.stop);
        }
    delete ctx;
}

extern "C" int etf_profile_enable(etf_ctx *ctx, int on)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->device < 0) return fail(ctx, ETF_ENOGPU, "host-only context");
    ctx->profile_on = on != 0;
    return ETF_OK;
}

extern "C" int etf_profile_read(etf_ctx *ctx, double *ms, int64_t *launches)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->device < 0) return fail(ctx, ETF_ENOGPU, "host-only context");
    if (!ms || !launches) return fail(ctx, ETF_EINVAL, "output pointer is null");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, hipStreamSynchronize((hipStream_t)ctx->stream));
    for (int i = 0; i < ETF_K_COUNT; ++i) {
        ms[i] = 0.0;
        launches[i] = 0;
    }
    for (auto &s : ctx->stamps) {
        float t = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&t, (hipEvent_t)s.start, (hipEvent_t)s.stop));
        ms[s.cls] += t;
        launches[s.cls] += 1;
        ctx->stamp_pool.push_back(s);
    }
    ctx->stamps.clear();
    return ETF_OK;
}

extern "C" int etf_set_stream(etf_ctx *ctx, void *hip_stream)
{
    if (!ctx) return ETF_EINVAL;
    ctx->stream = hip_stream;
    return ETF_OK;
}

static int need_device(const etf_ctx *ctx)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->device < 0) return fail(ctx, ETF_ENOGPU, "host-only context");
    return ETF_OK;
}

// =============================================================================================
// index upload
// =============================================================================================
extern "C" int etf_index_upload(etf_ctx *ctx, void *dev_buf, int64_t bytes)
{
    int rc = need_device(ctx);
    if (rc) return rc;
    if (!ctx->idx.built) return fail(ctx, ETF_ESTATE, "no index: call etf_index_build first");
    if (ctx->idx.device_built) return fail(ctx, ETF_ESTATE, "the index was built on the device and is resident already");
    if (!dev_buf) return fail(ctx, ETF_EINVAL, "device buffer is null");
    if (((uintptr_t)dev_buf & 255) != 0) return fail(ctx, ETF_EINVAL, "device buffer must be 256-byte aligned");
    if (bytes < ctx->lay.total) return fail(ctx, ETF_ENOMEM, "device buffer too small: %lld < %lld", (long long)bytes, (long long)ctx->lay.total);
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t st = (hipStream_t)ctx->stream;
    char *base = (char *)dev_buf;
    hipError_t first = hipSuccess;
    for_each_image_array(ctx, [&](int64_t off, const void *src, size_t n) {
        if (n == 0 || first != hipSuccess) return;
        first = hipMemcpyAsync(base + off, src, n, hipMemcpyHostToDevice, st);
    });
    HIP_TRY(ctx, first);
    HIP_TRY(ctx, hipStreamSynchronize(st));
    ctx->dev_base = base;
    ctx->last_flag_count = nullptr;
    return ETF_OK;
}

// =============================================================================================
// workspace plan
// =============================================================================================
namespace {

struct Plan {
    int mode = 0;
    bool search = false;
    int k = 0;
    int64_t tiles_total = 0;  // ceil(Q / 64)
    int64_t NT = 0;           // tiles per batch
    int64_t items = 0;        // candidates per query: N (flat) or distinct encodings
    int64_t S = 0;            // threshold sample size
    int gsize = 1;            // sample entries per group (only group minima are kept)
    int64_t ngroups = 0;      // ceil(S / gsize)
    uint32_t C = 0;           // candidate capacity per query
    bool use_tau = false;
    bool ctx_path = false;    // trees walked with the distance context in registers (no partial-sum tables)
    bool lds_path = false;    // search with every table slice in LDS: no result tables at all
    bool flat_lds = false;    // flat mode through the same kernels
    bool fx = false;          // the main pass of the LDS-resident search filters candidates in fixed point
    bool fx16 = false;        // ... on 16-bit tables (k_lds16)
    int64_t o_counter = 0, o_lutT = 0, o_gmin = 0, o_tau = 0, o_boff = 0, o_bm = 0, o_cnt = 0, o_flag = 0, o_cand = 0;
    int64_t o_part[ETF_MAX_M][ETF_MAX_M];
    int64_t o_leafp[ETF_MAX_M];
    int64_t total = 0;
};

int64_t al256(int64_t x) { return (x + 255) & ~(int64_t)255; }
int pow2_at_least_host(int n)
{
    int p = 1;
    while (p < n) p <<= 1;
    return p;
}
int tmax_class(int T);
int pick_G(int width, int K);
bool lds_eligible(int M, int K, int T, const int32_t *chunk_begin);

int make_plan(const etf_ctx *ctx, int64_t Q, int k, int mode, bool search, Plan &P, int64_t ws_cap = 0)
{
    if (ws_cap <= 0) ws_cap = ctx->opt.ws_cap_bytes;
    const HostIndex &ix = ctx->idx;
    if (!ix.built) return fail(ctx, ETF_ESTATE, "no index: call etf_index_build first");
    if (Q <= 0) return fail(ctx, ETF_EINVAL, "Q must be positive");
    if (mode != ETF_MODE_FLAT && mode != ETF_MODE_TREE && mode != ETF_MODE_FOREST)
        return fail(ctx, ETF_EINVAL, "unknown mode %d", mode);
    if (mode == ETF_MODE_TREE && ix.T != 1) return fail(ctx, ETF_ESTATE, "ETF_MODE_TREE needs an index built with T = 1 (it has T = %d)", ix.T);
    if (search && (k < 1 || k > ETF_MAX_TOPK || k > ix.N)) return fail(ctx, ETF_EINVAL, "need 1 <= k <= min(N, %d) (k=%d)", ETF_MAX_TOPK, k);
    P.mode = mode;
    P.search = search;
    P.k = k;
    P.tiles_total = (Q + QT - 1) / QT;
    const int M = ix.M, K = ix.K;
    P.items = mode == ETF_MODE_FLAT ? ix.N : ix.Nd;
    P.S = mode == ETF_MODE_FLAT ? ix.n_sample_pos : ix.n_sample_enc;
    if (search) {
        // The sample is cut into at least 1024 (256) and at least 2.5 k groups; the bound is the k-th smallest group
        // minimum, which lets through 1.05 to 1.3 times k items/S candidates per query (the more groups, the
        // closer the bound is to the k-th smallest sample; small groups also spread the sample pass over more waves).
        // (The table-based kernels take one group per wave: they keep 256.)
        const bool lds_kernels = ctx->opt.traversal == 2 &&
                                 (mode == ETF_MODE_FLAT ? lds_eligible(M, K, 1, nullptr) : lds_eligible(M, K, ix.T, ix.chunk_begin.data()));
        int64_t groups = lds_kernels ? 1024 : 256;
        while (groups < (int64_t)(2.5 * k) && groups < 4096) groups <<= 1;
        // (rounded up: at most `groups` groups, so that the sample pass's stretches of groups divide evenly among the
        // waves of its workgroups; 1025 groups instead of 1024 cost cfg2's pass 7 % and cfg4's 23 %)
        P.gsize = (int)std::max<int64_t>(1, (P.S + groups - 1) / groups);
        P.ngroups = (P.S + P.gsize - 1) / P.gsize;
        int64_t C = ctx->opt.cand_cap;
        if (C == 0) {
            int64_t expect = (int64_t)(1.3 * (double)k * (double)P.items / (double)std::max<int64_t>(P.S, 1));
            // The sample of the tree modes draws an encoding in proportion to the number of vectors that have it (the
            // bound counts vectors).  A query whose neighbourhood holds encodings of single vectors then sees up to
            // N / Nd times the candidates of one in a region of average duplication.
            if (mode != ETF_MODE_FLAT && ix.Nd > 0) expect = (int64_t)((double)expect * std::min(8.0, (double)ix.N / (double)ix.Nd));
            // the flat scan lists every copy of an encoding at or below the bound
            const int64_t copies = mode == ETF_MODE_FLAT ? 2 * ix.max_dup : 0;
            C = 4096;
            // (up to four million entries there: the batch of queries shrinks to keep the workspace under its cap)
            const int64_t limit = mode == ETF_MODE_FLAT ? (1 << 22) : (1 << 17);
            while (C < 3 * expect + 2048 + copies && C < limit) C <<= 1;
        }
        if (P.items <= C || P.ngroups < k) {  // few enough encodings: every one is a candidate, no bound needed
            P.use_tau = false;
            if (P.items > C) C = P.items;  // cannot bound without a large enough sample
        } else {
            P.use_tau = true;
        }
        P.C = (uint32_t)C;
    }
    // bytes per tile of 64 queries
    int64_t per_tile = (int64_t)M * K * QT * 4;
    // traversal 2 = every table slice in LDS, for searches on the shapes that kernel is built for; otherwise
    // it means the register-context kernels, like traversal 0
    P.lds_path = mode != ETF_MODE_FLAT && ctx->opt.traversal == 2 && lds_eligible(M, K, ix.T, ix.chunk_begin.data());
    P.flat_lds = mode == ETF_MODE_FLAT && ctx->opt.traversal == 2 && lds_eligible(M, K, 1, nullptr);
    // the fixed-point filter scales every table by its query's bound: it needs one (use_tau)
    // (not the flat scan: it lists every copy of an encoding, and copies tie exactly)
    P.fx = search && P.lds_path && P.use_tau && ctx->opt.lds_filter == 1 && !ctx->opt.force_fallback && !ix.has_term;
    // 16-bit tables: built for rows of 64 and 32 bytes (M = 8 and M = 16 at K = 256); other shapes keep the float32 sums
    P.fx16 = search && P.lds_path && P.use_tau && ctx->opt.lds_filter == 2 && !ctx->opt.force_fallback && !ix.has_term &&
             (M == 8 || M == 16) && std::max(2, pick_G(M, K)) == (M == 8 ? 4 : 8);
    P.ctx_path = !P.lds_path && tmax_class(ix.T) != 0 && mode != ETF_MODE_FLAT && ctx->opt.traversal != 1;
    for (int t = 1; t < ix.T; ++t)  // the register-context kernels address a tree's result table with 32-bit offsets
        if (ix.tree[t].U >= ((int64_t)1 << 24)) P.ctx_path = false;
    if (ix.Nd >= ((int64_t)1 << 26)) P.ctx_path = false;  // its candidate records keep the item in 26 bits
    if (mode != ETF_MODE_FLAT && !P.lds_path)
        for (int t = P.ctx_path ? 1 : 0; t < ix.T; ++t) {
            const HostTree &tr = ix.tree[t];
            if (!P.ctx_path)
                for (int l = 0; l + 1 < tr.D; ++l) per_tile += al256(tr.nI[l] * QT * 4);
            per_tile += al256(tr.U * QT * 4);
        }
    if (search) {
        if (P.use_tau) per_tile += al256(P.ngroups * QT * 4);
        per_tile += (int64_t)QT * (12 + (int64_t)P.C * 8);
    }
    int64_t nt = ws_cap / std::max<int64_t>(per_tile + 4096, 1);
    P.NT = std::max<int64_t>(1, std::min<int64_t>(nt, P.tiles_total));
    // offsets
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        int64_t o = off;
        off = al256(off + bytes);
        return o;
    };
    P.o_counter = take(256);
    P.o_lutT = take(P.NT * M * K * QT * 4);
    if (mode != ETF_MODE_FLAT && !P.lds_path)
        for (int t = P.ctx_path ? 1 : 0; t < ix.T; ++t) {
            const HostTree &tr = ix.tree[t];
            if (!P.ctx_path)
                for (int l = 0; l + 1 < tr.D; ++l) P.o_part[t][l] = take(P.NT * tr.nI[l] * QT * 4);
            P.o_leafp[t] = take(P.NT * tr.U * QT * 4);
        }
    if (search) {
        if (P.use_tau) P.o_gmin = take(P.NT * P.ngroups * QT * 4);
        P.o_tau = take(P.NT * QT * 4);
        P.o_boff = take(P.NT * QT * 4);
        P.o_bm = take(P.NT * M * QT * 4);
        P.o_cnt = take(P.NT * QT * 4);
        P.o_flag = take(P.NT * QT * 4);
        P.o_cand = take(P.NT * QT * (int64_t)P.C * 8);
    }
    P.total = off;
    return ETF_OK;
}

// choose the number of workgroups along x so that a launch has a few thousand workgroups in total
int64_t blocks_for(int64_t n, int64_t min_items_per_block, int64_t other_dims)
{
    int64_t want = std::max<int64_t>(1, 4096 / std::max<int64_t>(other_dims, 1));
    int64_t b = (n + min_items_per_block - 1) / min_items_per_block;
    return std::max<int64_t>(1, std::min<int64_t>(b, want));
}

// Workgroups per sub-tile of queries for the LDS-resident kernels.  A CU holds one workgroup (its tables fill the
// LDS), so a launch of W * bx workgroups runs in ceil(W * bx / 256) rounds, and each round has a fixed cost beside
// its nitems / bx items: the workgroup's start, staging the tables, the first record loads, waves that finish at
// different times while the LDS cannot be handed on (measured: 6 us, the time of about 5000 items at M = 8).
// The cost of a choice is rounds * (5000 + nitems / bx), in items.  Few large workgroups win unless they leave
// CUs idle.
int64_t lds_blocks_for(int64_t W, int64_t nitems, int64_t min_bx, int64_t least_items = 4096)
{
    const int64_t cus = 256, stage_items = 5000;
    int64_t best = min_bx, best_cost = -1;
    const int64_t max_bx = std::max(min_bx, (nitems + least_items - 1) / least_items);  // a workgroup of 16 waves wants a few thousand items
    for (int64_t bx = min_bx; bx <= max_bx && bx < min_bx + 256; ++bx) {
        const int64_t rounds = (W * bx + cus - 1) / cus;
        const int64_t cost = rounds * (stage_items + (nitems + bx - 1) / bx);
        if (best_cost < 0 || cost < best_cost) {
            best = bx;
            best_cost = cost;
        }
        if (W * bx >= 16 * cus) break;  // beyond 16 rounds only the staging grows
    }
    return best;
}

int pick_G(int width, int K)
{
    int G = 1;
    while (G < 16 && (int64_t)width * K * (WAVE / G) * 4 > LDS_BUDGET) G <<= 1;
    return G;
}

template <class F>
int set_lds(const etf_ctx *ctx, F kernel, size_t bytes)
{
    if (bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return fail(ctx, ETF_EHIP, "hipFuncSetAttribute(%zu bytes of LDS): %s", bytes, hipGetErrorString(e));
    }
    return ETF_OK;
}

// ---- launch helpers --------------------------------------------------------------------------

int launch_lut(etf_ctx *ctx, const float *queries, int64_t Q, int64_t q0, int64_t tiles, float *lutT, float *lut_public)
{
    dim3 grid((unsigned)tiles, (unsigned)ctx->M);
    // one wave per workgroup and 32 codewords per wave for the matrix-core kernel (option lut_narrow_below: always, by
    // default): the launch spreads over more compute units and more waves hide each other's sweeps and stores
    const bool narrow = tiles * ctx->M < ctx->opt.lut_narrow_below;
    const dim3 mgrid((unsigned)tiles, (unsigned)ctx->M, narrow ? (unsigned)((ctx->K + 31) / 32) : 1u), mblock(narrow ? 64 : 256);
    ChunkOrder ord;
    for (int j = 0; j < ETF_MAX_M; ++j) ord.src[j] = (uint8_t)((size_t)j < ctx->idx.order.size() ? ctx->idx.order[j] : j);
    ProfScope prof(ctx, ETF_K_LUT);
    if (ctx->opt.metric == 1 && ctx->opt.lut_kernel == 0) {
        const float *cb = reinterpret_cast<const float *>(ctx->dev_base + ctx->lay.codebooks);
        if (narrow)
            hipLaunchKernelGGL((k_lut_mfma<true, 1>), mgrid, mblock, 0, (hipStream_t)ctx->stream, queries, Q, q0, ctx->d, ctx->M, ctx->K,
                               cb, nullptr, nullptr, nullptr, ctx->dsp, lutT, lut_public, ord);
        else
            hipLaunchKernelGGL((k_lut_mfma<true, 2>), mgrid, mblock, 0, (hipStream_t)ctx->stream, queries, Q, q0, ctx->d, ctx->M, ctx->K,
                               cb, nullptr, nullptr, nullptr, ctx->dsp, lutT, lut_public, ord);
        LAUNCH_CHECK(ctx, "k_lut_mfma");
    } else if (ctx->opt.metric == 1) {
        const float *cb = reinterpret_cast<const float *>(ctx->dev_base + ctx->lay.codebooks);
        hipLaunchKernelGGL(k_lut_direct<true>, grid, dim3(256), 0, (hipStream_t)ctx->stream, queries, Q, q0, ctx->d, ctx->M,
                           ctx->K, cb, lutT, lut_public, ord);
        LAUNCH_CHECK(ctx, "k_lut_direct");
    } else if (ctx->opt.lut_kernel == 0) {
        const float *cbc = reinterpret_cast<const float *>(ctx->dev_base + ctx->lay.cb_centered);
        const float *cbn = reinterpret_cast<const float *>(ctx->dev_base + ctx->lay.cb_norm);
        const float *cbm = reinterpret_cast<const float *>(ctx->dev_base + ctx->lay.cb_mean);
        const float *cb = reinterpret_cast<const float *>(ctx->dev_base + ctx->lay.codebooks);
        if (narrow)
            hipLaunchKernelGGL((k_lut_mfma<false, 1>), mgrid, mblock, 0, (hipStream_t)ctx->stream, queries, Q, q0, ctx->d, ctx->M, ctx->K,
                               cb, cbc, cbn, cbm, ctx->dsp, lutT, lut_public, ord);
        else
            hipLaunchKernelGGL((k_lut_mfma<false, 2>), mgrid, mblock, 0, (hipStream_t)ctx->stream, queries, Q, q0, ctx->d, ctx->M, ctx->K,
                               cb, cbc, cbn, cbm, ctx->dsp, lutT, lut_public, ord);
        LAUNCH_CHECK(ctx, "k_lut_mfma");
    } else {
        const float *cb = reinterpret_cast<const float *>(ctx->dev_base + ctx->lay.codebooks);
        hipLaunchKernelGGL(k_lut_direct<false>, grid, dim3(256), 0, (hipStream_t)ctx->stream, queries, Q, q0, ctx->d, ctx->M,
                           ctx->K, cb, lutT, lut_public, ord);
        LAUNCH_CHECK(ctx, "k_lut_direct");
    }
    return ETF_OK;
}

template <int G>
int launch_leaf_g(etf_ctx *ctx, int ndw, dim3 grid, dim3 block, size_t lds, const uint8_t *lcodes, int width,
                  const uint32_t *lparent, const uint32_t *lrow, int64_t n, const float *prev, int64_t nprev, float *out,
                  int64_t U, const float *lutT, int m0, int per_block)
{
    hipStream_t st = (hipStream_t)ctx->stream;
    const int M = ctx->M, K = ctx->K;
    ProfScope prof(ctx, ETF_K_LEAF);
#define LEAF_CASE(NDW)                                                                                         \
    case NDW: {                                                                                                \
        int rc = set_lds(ctx, k_leaf<G, NDW>, lds);                                                            \
        if (rc) return rc;                                                                                     \
        hipLaunchKernelGGL((k_leaf<G, NDW>), grid, block, lds, st, lcodes, width, lparent, lrow, n, prev, nprev, \
                           out, U, lutT, M, K, m0, per_block);                                                 \
        break;                                                                                                 \
    }
    switch (ndw) {
        LEAF_CASE(1)
        LEAF_CASE(2)
        LEAF_CASE(3)
        LEAF_CASE(4)
        default: return fail(ctx, ETF_EINVAL, "leaf record of %d words", ndw);
    }
#undef LEAF_CASE
    LAUNCH_CHECK(ctx, "k_leaf");
    return ETF_OK;
}

// all levels and leaf buckets of every tree for `tiles` tiles: fills the per-tree result tables
int launch_trees(etf_ctx *ctx, const Plan &P, char *ws, int64_t tiles)
{
    const HostIndex &ix = ctx->idx;
    const DevLayout &L = ctx->lay;
    hipStream_t st = (hipStream_t)ctx->stream;
    const float *lutT = reinterpret_cast<const float *>(ws + P.o_lutT);
    const int M = ix.M, K = ix.K;
    for (int t = 0; t < ix.T; ++t) {
        const HostTree &tr = ix.tree[t];
        const DevTreeLayout &TL = L.tree[t];
        // internal levels, top down
        for (int l = 0; l + 1 < tr.D; ++l) {
            const int64_t n = tr.nI[l];
            if (n == 0) break;  // no internal node at this level: none below either
            const int64_t bx = blocks_for(n, 4 * 32, tiles);
            const int per_wave = (int)((n + bx * 4 - 1) / (bx * 4));
            const float *prev = l > 0 ? reinterpret_cast<const float *>(ws + P.o_part[t][l - 1]) : nullptr;
            const int64_t nprev = l > 0 ? tr.nI[l - 1] : 0;
            ProfScope prof(ctx, ETF_K_LEVEL);
            hipLaunchKernelGGL(k_level, dim3((unsigned)bx, (unsigned)tiles), dim3(256), 0, st,
                               reinterpret_cast<const uint8_t *>(ctx->dev_base + TL.icode[l]),
                               reinterpret_cast<const uint32_t *>(ctx->dev_base + TL.iparent[l]), n, prev, nprev,
                               reinterpret_cast<float *>(ws + P.o_part[t][l]), lutT, M, K, tr.c0 + l, per_wave);
            LAUNCH_CHECK(ctx, "k_level");
        }
        // leaf buckets
        for (int l = 0; l < tr.D; ++l) {
            const HostBucket &B = tr.bucket[l];
            const int64_t n = tr.nL[l];
            if (n == 0) continue;
            const float *prev = l > 0 ? reinterpret_cast<const float *>(ws + P.o_part[t][l - 1]) : nullptr;
            const int64_t nprev = l > 0 ? tr.nI[l - 1] : 0;
            const uint8_t *lc = reinterpret_cast<const uint8_t *>(ctx->dev_base + TL.lcodes[l]);
            const uint32_t *lp = reinterpret_cast<const uint32_t *>(ctx->dev_base + TL.lparent[l]);
            const uint32_t *lr = reinterpret_cast<const uint32_t *>(ctx->dev_base + TL.lrow[l]);
            float *out = reinterpret_cast<float *>(ws + P.o_leafp[t]);
            if (B.width <= 2) {  // short leaves: table rows straight from L2, no LDS staging
                const int64_t bx = blocks_for(n, 4 * 64, tiles);
                int per_wave = (int)((n + bx * 4 - 1) / (bx * 4));
                per_wave = (per_wave + 63) & ~63;
                const int64_t bx2 = (n + (int64_t)per_wave * 4 - 1) / ((int64_t)per_wave * 4);
                ProfScope prof(ctx, ETF_K_LEAF);
                if (B.width == 1)
                    hipLaunchKernelGGL((k_leaf_short<1>), dim3((unsigned)bx2, (unsigned)tiles), dim3(256), 0, st, lc, lp, lr, n,
                                       prev, nprev, out, tr.U, lutT, M, K, tr.c0 + l, per_wave);
                else
                    hipLaunchKernelGGL((k_leaf_short<2>), dim3((unsigned)bx2, (unsigned)tiles), dim3(256), 0, st, lc, lp, lr, n,
                                       prev, nprev, out, tr.U, lutT, M, K, tr.c0 + l, per_wave);
                LAUNCH_CHECK(ctx, "k_leaf_short");
                continue;
            }
            const int G = pick_G(B.width, K);
            const size_t lds = (size_t)B.width * K * (WAVE / G) * 4;
            const int64_t bx = blocks_for(n, 2048, tiles * G);
            const int per_block = (int)((n + bx - 1) / bx);
            dim3 grid((unsigned)bx, (unsigned)G, (unsigned)tiles), block(512);
            int rc;
            switch (G) {
                case 1: rc = launch_leaf_g<1>(ctx, B.stride / 4, grid, block, lds, lc, B.width, lp, lr, n, prev, nprev, out, tr.U, lutT, tr.c0 + l, per_block); break;
                case 2: rc = launch_leaf_g<2>(ctx, B.stride / 4, grid, block, lds, lc, B.width, lp, lr, n, prev, nprev, out, tr.U, lutT, tr.c0 + l, per_block); break;
                case 4: rc = launch_leaf_g<4>(ctx, B.stride / 4, grid, block, lds, lc, B.width, lp, lr, n, prev, nprev, out, tr.U, lutT, tr.c0 + l, per_block); break;
                case 8: rc = launch_leaf_g<8>(ctx, B.stride / 4, grid, block, lds, lc, B.width, lp, lr, n, prev, nprev, out, tr.U, lutT, tr.c0 + l, per_block); break;
                default: rc = fail(ctx, ETF_EINVAL, "no kernel for %d leaves per wave", G);
            }
            if (rc) return rc;
        }
    }
    return ETF_OK;
}

void fill_reduce_args(const etf_ctx *ctx, const Plan &P, char *ws, ReduceArgs &r)
{
    const HostIndex &ix = ctx->idx;
    memset(&r, 0, sizeof r);
    r.T = ix.T;
    for (int t = 0; t < ix.T; ++t) {
        r.leafp[t] = reinterpret_cast<const float *>(ws + P.o_leafp[t]);
        r.leaf_of[t] = ctx->lay.tree[t].leaf_of >= 0 ? reinterpret_cast<const uint32_t *>(ctx->dev_base + ctx->lay.tree[t].leaf_of) : nullptr;
        r.U[t] = ix.tree[t].U;
    }
    // padding slots up to the kernel's compile-time tree count: valid, cached, and not added
    for (int t = ix.T; t < ETF_MAX_M; ++t) {
        r.leafp[t] = r.leafp[0];
        r.leaf_of[t] = r.leaf_of[0];
        r.U[t] = r.U[0];
    }
}

// ---- register-context traversal ----------------------------------------------------------------

int tmax_class(int T) { return T <= 1 ? 1 : T <= 2 ? 2 : T <= 4 ? 4 : 0; }

// The fused tree-0 kernel is instantiated for up to 4 trees; other shapes (and the explicit option) use
// the level-synchronous kernels.

// result tables of trees 1 .. T-1 (tree 0 is evaluated inside the fused kernel)
int launch_trees_ctx(etf_ctx *ctx, const Plan &P, char *ws, int64_t tiles)
{
    const HostIndex &ix = ctx->idx;
    hipStream_t st = (hipStream_t)ctx->stream;
    const float *lutT = reinterpret_cast<const float *>(ws + P.o_lutT);
    for (int t = 1; t < ix.T; ++t) {
        const HostTree &tr = ix.tree[t];
        const uint32_t *codes = reinterpret_cast<const uint32_t *>(ctx->dev_base + ctx->lay.tree[t].rec);
        float *out = reinterpret_cast<float *>(ws + P.o_leafp[t]);
        // 16 waves per workgroup share the staged slices; about 2048 workgroups per launch
        const int64_t bx = blocks_for(tr.U, 16 * 64 * 4, tiles * 2);
        int per_wave = (int)((tr.U + bx * 16 - 1) / (bx * 16));
        per_wave = (per_wave + 63) & ~63;
        const int64_t bx2 = (tr.U + (int64_t)per_wave * 16 - 1) / ((int64_t)per_wave * 16);
        const dim3 grid((unsigned)bx2, (unsigned)tiles), block(1024);
        ProfScope prof(ctx, ETF_K_LEAF);
#define TREE_CASE(DT, NDW, NL)                                                                                   \
    case DT: {                                                                                                   \
        const size_t lds = (size_t)NL * ix.K * QT * 4;                                                           \
        int rc = set_lds(ctx, k_tree_ctx<DT, NDW, NL, CUB>, lds);                                                     \
        if (rc) return rc;                                                                                       \
        hipLaunchKernelGGL((k_tree_ctx<DT, NDW, NL, CUB>), grid, block, lds, st, codes, tr.U, out, lutT, ix.M, ix.K,  \
                           tr.c0, tr.D, per_wave);                                                               \
        break;                                                                                                   \
    }
        switch (depth_class(tr.D)) {
            TREE_CASE(1, 1, 1)
            TREE_CASE(2, 1, 2)
            TREE_CASE(4, 1, 2)
            TREE_CASE(8, 2, 2)
            TREE_CASE(16, 4, 2)
            default: return fail(ctx, ETF_EINVAL, "tree depth %d", tr.D);
        }
#undef TREE_CASE
        LAUNCH_CHECK(ctx, "k_tree_ctx");
    }
    return ETF_OK;
}

void fill_fused_args(const etf_ctx *ctx, const Plan &P, char *ws, ReduceArgs &r)
{
    const HostIndex &ix = ctx->idx;
    memset(&r, 0, sizeof r);
    r.T = ix.T;
    for (int t = 1; t < ix.T; ++t) {
        r.leafp[t] = reinterpret_cast<const float *>(ws + P.o_leafp[t]);
        r.leaf_of[t] = reinterpret_cast<const uint32_t *>(ctx->dev_base + ctx->lay.tree[t].leaf_of);
        r.U[t] = ix.tree[t].U;
    }
    // padding slots up to the kernel's compile-time tree count: valid, cached, and not added
    for (int t = std::max(ix.T, 2); t < ETF_MAX_M; ++t) {
        r.leafp[t] = r.leafp[1];
        r.leaf_of[t] = r.leaf_of[1];
        r.U[t] = r.U[1];
    }
}

template <int MODE, int DT, int NDW>
int launch_fused_d(etf_ctx *ctx, const Plan &P, char *ws, const ReduceArgs &r, int64_t nitems, const uint32_t *map,
                   const OutArgs &o, dim3 grid, dim3 block, int per_wave)
{
    constexpr int NL = MODE == OUT_ALLPAIRS ? 0 : (DT >= 2 ? 2 : 1);
    const HostIndex &ix = ctx->idx;
    hipStream_t st = (hipStream_t)ctx->stream;
    const float *lutT = reinterpret_cast<const float *>(ws + P.o_lutT);
    const uint32_t *codes0 = reinterpret_cast<const uint32_t *>(ctx->dev_base + ctx->lay.rec0);
    const int D0 = ix.tree[0].D;
    const size_t lds = (size_t)NL * ix.K * QT * 4;
#define FUSED_CASE(TM)                                                                                              \
    case TM: {                                                                                                      \
        int rc = set_lds(ctx, k_fused<MODE, DT, NDW, TM, NL, CUB>, lds);                                                 \
        if (rc) return rc;                                                                                          \
        hipLaunchKernelGGL((k_fused<MODE, DT, NDW, TM, NL, CUB>), grid, block, lds, st, codes0, D0, lutT, ix.M, ix.K, r, \
                           nitems, map, per_wave, o);                                                               \
        break;                                                                                                      \
    }
    switch (tmax_class(ix.T)) {
        FUSED_CASE(1)
        FUSED_CASE(2)
        FUSED_CASE(4)
        default: return fail(ctx, ETF_EINVAL, "no fused kernel for %d trees", ix.T);
    }
#undef FUSED_CASE
    LAUNCH_CHECK(ctx, "k_fused");
    return ETF_OK;
}

template <int MODE>
int launch_fused(etf_ctx *ctx, const Plan &P, char *ws, const ReduceArgs &r, int64_t nitems, const uint32_t *map,
                 int64_t tiles, const OutArgs &o)
{
    if (nitems == 0) return ETF_OK;
    // all-pairs output is transposed through a per-wave LDS tile: 4 waves per workgroup there, 16 elsewhere
    const int wpb = MODE == OUT_ALLPAIRS ? 4 : 16;
    int per_wave;
    if (MODE == OUT_SAMPLE) {
        per_wave = o.gsize;  // one sample group per wave
    } else {
        const int64_t bx = blocks_for(nitems, wpb * 64 * 4, tiles * (MODE == OUT_ALLPAIRS ? 1 : 2));
        per_wave = (int)((nitems + bx * wpb - 1) / (bx * wpb));
        per_wave = (per_wave + 63) & ~63;
    }
    const int64_t bx2 = (nitems + (int64_t)per_wave * wpb - 1) / ((int64_t)per_wave * wpb);
    const dim3 grid((unsigned)bx2, (unsigned)tiles), block(wpb * 64);
    ProfScope prof(ctx, MODE == OUT_SAMPLE ? ETF_K_SAMPLE : ETF_K_REDUCE);
    switch (depth_class(ctx->idx.tree[0].D)) {
        case 1: return launch_fused_d<MODE, 1, 1>(ctx, P, ws, r, nitems, map, o, grid, block, per_wave);
        case 2: return launch_fused_d<MODE, 2, 1>(ctx, P, ws, r, nitems, map, o, grid, block, per_wave);
        case 4: return launch_fused_d<MODE, 4, 1>(ctx, P, ws, r, nitems, map, o, grid, block, per_wave);
        case 8: return launch_fused_d<MODE, 8, 2>(ctx, P, ws, r, nitems, map, o, grid, block, per_wave);
        case 16: return launch_fused_d<MODE, 16, 4>(ctx, P, ws, r, nitems, map, o, grid, block, per_wave);
        default: return fail(ctx, ETF_EINVAL, "tree depth %d", ctx->idx.tree[0].D);
    }
}

template <int MODE>
int launch_reduce(etf_ctx *ctx, const ReduceArgs &r, int64_t nitems, const uint32_t *map, int64_t tiles, const OutArgs &o)
{
    if (nitems == 0) return ETF_OK;
    int per_wave;
    if (MODE == OUT_SAMPLE) {
        per_wave = o.gsize;  // one sample group per wave
    } else {
        const int64_t bx = blocks_for(nitems, 4 * 64, tiles);
        per_wave = (int)((nitems + bx * 4 - 1) / (bx * 4));
        per_wave = (per_wave + 63) & ~63;  // whole 64-item chunks per wave
    }
    const int64_t bx2 = (nitems + (int64_t)per_wave * 4 - 1) / ((int64_t)per_wave * 4);
    const dim3 grid((unsigned)bx2, (unsigned)tiles), block(256);
    hipStream_t st = (hipStream_t)ctx->stream;
    ProfScope prof(ctx, MODE == OUT_SAMPLE ? ETF_K_SAMPLE : ETF_K_REDUCE);
    if (r.T <= 1) hipLaunchKernelGGL((k_reduce<MODE, 1>), grid, block, 0, st, r, nitems, map, per_wave, o);
    else if (r.T <= 2) hipLaunchKernelGGL((k_reduce<MODE, 2>), grid, block, 0, st, r, nitems, map, per_wave, o);
    else if (r.T <= 4) hipLaunchKernelGGL((k_reduce<MODE, 4>), grid, block, 0, st, r, nitems, map, per_wave, o);
    else if (r.T <= 8) hipLaunchKernelGGL((k_reduce<MODE, 8>), grid, block, 0, st, r, nitems, map, per_wave, o);
    else hipLaunchKernelGGL((k_reduce<MODE, 16>), grid, block, 0, st, r, nitems, map, per_wave, o);
    LAUNCH_CHECK(ctx, "k_reduce");
    return ETF_OK;
}

// Every table slice of a sub-tile in LDS: which shapes the kernel is built for.  Trees must be T equal
// groups of chunks (chunk_begin == nullptr: a single group).
bool lds_eligible(int M, int K, int T, const int32_t *chunk_begin)
{
    if (M != 4 && M != 8 && M != 16) return false;
    if (T < 1 || T > M || M % T != 0) return false;
    const int D = M / T;  // trees of whole groups of four chunks, or of one or two chunks inside a pair
    if (D >= 4 ? D % 4 != 0 : (D != 1 && D != 2)) return false;
    if (chunk_begin)
        for (int t = 0; t <= T; ++t)
            if (chunk_begin[t] != t * (M / T)) return false;
    const int G = std::max(2, pick_G(M, K));
    if (G > 8) return false;
    return M % lds_chunks_per_line(G) == 0;  // whole lines of 4 (8 at eight queries per sub-tile) chunks
}

template <int MODE, bool CTX, bool FX = false, bool TERM = false>
int launch_lds(etf_ctx *ctx, const Plan &P, char *ws, const uint32_t *rec, int64_t nitems, const uint32_t *map, int T,
               int64_t tiles, const OutArgs &o, int cls)
{
    if (nitems == 0) return ETF_OK;
    const int M = ctx->M, K = ctx->K;
    const int G = std::max(2, pick_G(M, K));
    const size_t lds = lds_table_bytes(G, M, K) + lds_aux_bytes(MODE == OUT_FILTER);
    const int IPS = LDS_V * G;  // items per wave step
    // The kernels are built for trees of at least four chunks (1, 2 or 4 trees); shorter trees lie inside the
    // pairs of a group of four, whose sum is formed the same way whatever the trees: they run as trees of four.
    if (M / T < 4) T = M / 4;
    if (FX) T = 1;  // integer sums do not depend on the order of additions: one instance serves every forest
    int64_t bx;
    int per_block = 0;
    if (MODE == OUT_SAMPLE) {
        // every workgroup stages the whole table set: give each wave at least two stretches of IPS sample groups
        bx = blocks_for(o.ngroups, 2 * 16 * IPS, tiles * G);
    } else {
        // item numbers inside a workgroup's share travel in 26 bits
        if (MODE == OUT_ALLPAIRS) {
            // sub-tiles past the last query end at once: only the live ones share the compute units, and a small
            // batch should fill them in one round
            const int64_t Qs = WAVE / G, live = std::min<int64_t>(tiles * G, (o.nq + Qs - 1) / Qs);
            const bool few = live * ((nitems + 4095) / 4096) < 256;  // would leave compute units idle
            bx = lds_blocks_for(std::max<int64_t>(live, 1), nitems, (nitems >> 25) + 1, few ? 1024 : 4096);
        } else {
            bx = lds_blocks_for(tiles * G, nitems, (nitems >> 25) + 1);
        }
        if (ctx->opt.lds_blocks > 0) bx = std::max<int64_t>(ctx->opt.lds_blocks, (nitems >> 25) + 1);
        per_block = (int)((nitems + bx - 1) / bx);
    }
    dim3 grid((unsigned)bx, (unsigned)G, (unsigned)tiles);
    hipStream_t st = (hipStream_t)ctx->stream;
    const float *lutT = reinterpret_cast<const float *>(ws + P.o_lutT);
    ProfScope prof(ctx, cls);
    bool done = false;
#define LDS_CASE(GG, MM4, TT)                                                                                  \
    if constexpr ((CTX || MODE != OUT_FILTER || TT == 1) && (!FX || TT == 1) && (4 * MM4) % lds_chunks_per_line(GG) == 0) {                         \
        if (!done && G == GG && M == 4 * MM4 && T == TT) {                                                     \
            int rc = set_lds(ctx, k_lds<GG, MM4, TT, MODE, CTX, FX, TERM>, lds);                                     \
            if (rc) return rc;                                                                                 \
            hipLaunchKernelGGL((k_lds<GG, MM4, TT, MODE, CTX, FX, TERM>), grid, dim3(1024), lds, st, rec, nitems, map, lutT, K, \
                               per_block, o);                                                                  \
            done = true;                                                                                       \
        }                                                                                                      \
    }
#define LDS_CASES(GG) LDS_CASE(GG, 1, 1) LDS_CASE(GG, 2, 1) LDS_CASE(GG, 2, 2) LDS_CASE(GG, 4, 1) LDS_CASE(GG, 4, 2) \
    LDS_CASE(GG, 4, 4)
    LDS_CASES(2) LDS_CASES(4) LDS_CASES(8)
#undef LDS_CASES
#undef LDS_CASE
    if (!done) return fail(ctx, ETF_EINVAL, "no LDS-resident kernel for M=%d K=%d T=%d", M, K, T);
    LAUNCH_CHECK(ctx, "k_lds");
    return ETF_OK;
}

// the filter pass on 16-bit tables (see k_lds16)
int launch_lds16(etf_ctx *ctx, const Plan &P, char *ws, const uint32_t *rec, int64_t nitems, int64_t tiles, const OutArgs &o)
{
    if (nitems == 0) return ETF_OK;
    const int M = ctx->M, K = ctx->K;
    const int G = std::max(2, pick_G(M, K));
    const size_t lds = lds_table_bytes(G, M, K) + lds16_aux_bytes();
    int64_t bx = lds_blocks_for(tiles * (G / 2), nitems, (nitems >> 25) + 1);
    if (ctx->opt.lds_blocks > 0) bx = std::max<int64_t>(ctx->opt.lds_blocks, (nitems >> 25) + 1);
    const int per_block = (int)((nitems + bx - 1) / bx);
    dim3 grid((unsigned)bx, (unsigned)(G / 2), (unsigned)tiles);
    hipStream_t st = (hipStream_t)ctx->stream;
    const float *lutT = reinterpret_cast<const float *>(ws + P.o_lutT);
    ProfScope prof(ctx, ETF_K_LDS16);
    int rc;
    const bool cx = ctx->opt.lds16_context != 0;
    if (M == 8 && cx) {
        if ((rc = set_lds(ctx, k_lds16<4, 2, true>, lds))) return rc;
        hipLaunchKernelGGL((k_lds16<4, 2, true>), grid, dim3(1024), lds, st, rec, nitems, lutT, K, per_block, o);
    } else if (M == 8) {
        if ((rc = set_lds(ctx, k_lds16<4, 2, false>, lds))) return rc;
        hipLaunchKernelGGL((k_lds16<4, 2, false>), grid, dim3(1024), lds, st, rec, nitems, lutT, K, per_block, o);
    } else if (M == 16 && cx) {
        if ((rc = set_lds(ctx, k_lds16<8, 4, true>, lds))) return rc;
        hipLaunchKernelGGL((k_lds16<8, 4, true>), grid, dim3(1024), lds, st, rec, nitems, lutT, K, per_block, o);
    } else if (M == 16) {
        if ((rc = set_lds(ctx, k_lds16<8, 4, false>, lds))) return rc;
        hipLaunchKernelGGL((k_lds16<8, 4, false>), grid, dim3(1024), lds, st, rec, nitems, lutT, K, per_block, o);
    } else {
        return fail(ctx, ETF_EINVAL, "no 16-bit filter kernel for M=%d", M);
    }
    LAUNCH_CHECK(ctx, "k_lds16");
    return ETF_OK;
}

template <int MODE>
int launch_flat(etf_ctx *ctx, const Plan &P, char *ws, int64_t nitems, const uint32_t *sample, int64_t tiles, const OutArgs &o)
{
    if (nitems == 0) return ETF_OK;
    const int M = ctx->M, K = ctx->K;
    const int G = pick_G(M, K);
    const size_t lds = (size_t)M * K * (WAVE / G) * 4;
    // sample mode: every (wave, lane group) of the 8-wave block owns whole sample groups
    const int64_t bx = MODE == OUT_SAMPLE ? blocks_for(o.ngroups, 8 * G, tiles * G) : blocks_for(nitems, 4096, tiles * G);
    const int per_block = (int)((nitems + bx - 1) / bx);
    dim3 grid((unsigned)bx, (unsigned)G, (unsigned)tiles), block(512);
    hipStream_t st = (hipStream_t)ctx->stream;
    const uint8_t *codes = reinterpret_cast<const uint8_t *>(ctx->dev_base + ctx->lay.codes);
    const float *lutT = reinterpret_cast<const float *>(ws + P.o_lutT);
    if constexpr (MODE != OUT_ALLPAIRS)
        if (P.flat_lds) {
            // the sample's codes are stored side by side in sample order: no indirection
            const uint8_t *rec = MODE == OUT_SAMPLE ? reinterpret_cast<const uint8_t *>(ctx->dev_base + ctx->lay.sample_pos_codes) : codes;
            if (MODE == OUT_FILTER && ctx->idx.has_term)
                return launch_lds<MODE, false, false, MODE == OUT_FILTER>(ctx, P, ws, reinterpret_cast<const uint32_t *>(rec), nitems, nullptr,
                                                                          1, tiles, o, ETF_K_FLAT);
            return launch_lds<MODE, false>(ctx, P, ws, reinterpret_cast<const uint32_t *>(rec), nitems, nullptr, 1, tiles, o,
                                           MODE == OUT_SAMPLE ? ETF_K_SAMPLE : ETF_K_FLAT);
        }
    ProfScope prof(ctx, MODE == OUT_SAMPLE ? ETF_K_SAMPLE : ETF_K_FLAT);
#define FLAT_CASE(GG)                                                                                     \
    case GG: {                                                                                               \
        int rc = set_lds(ctx, k_flat<GG, MODE>, lds);                                                        \
        if (rc) return rc;                                                                                   \
        hipLaunchKernelGGL((k_flat<GG, MODE>), grid, block, lds, st, codes, nitems, sample, lutT, M, K, per_block, o); \
        break;                                                                                               \
    }
    switch (G) {
        FLAT_CASE(1)
        FLAT_CASE(2)
        FLAT_CASE(4)
        FLAT_CASE(8)
        default: return fail(ctx, ETF_EINVAL, "no kernel for %d encodings per wave", G);
    }
#undef FLAT_CASE
    LAUNCH_CHECK(ctx, "k_flat");
    return ETF_OK;
}

int check_ready(etf_ctx *ctx, const void *queries, const void *ws)
{
    int rc = need_device(ctx);
    if (rc) return rc;
    if (!ctx->idx.built) return fail(ctx, ETF_ESTATE, "no index: call etf_index_build first");
    if (!ctx->dev_base) return fail(ctx, ETF_ESTATE, "index not on the device: call etf_index_upload first");
    if (!queries) return fail(ctx, ETF_EINVAL, "queries pointer is null");
    if (!ws) return fail(ctx, ETF_EINVAL, "workspace pointer is null");
    if (((uintptr_t)ws & 255) != 0) return fail(ctx, ETF_EINVAL, "workspace must be 256-byte aligned");
    return ETF_OK;
}

}  // namespace

// plain streaming kernels over the caller's buffers: the memory ceilings a benchmark quotes beside the traversal
extern "C" int etf_probe_bandwidth(etf_ctx *ctx, int kind, void *a, void *b, int64_t bytes)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->device < 0) return fail(ctx, ETF_ENOGPU, "host-only context");
    if (!a || !b || bytes < 65536 || (bytes & 255) != 0 || (((uintptr_t)a | (uintptr_t)b) & 255) != 0)
        return fail(ctx, ETF_EINVAL, "probe buffers must be 256-byte aligned and a multiple of 256 bytes, at least 64 KiB");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t st = (hipStream_t)ctx->stream;
    const unsigned grid = 256 * 16;  // sixteen workgroups of 256 threads per compute unit; b must hold 4 bytes per workgroup
    const int64_t n16 = bytes / 16, nrows = bytes / 256;
    switch (kind) {
        case ETF_PROBE_READ: hipLaunchKernelGGL(k_probe_read, dim3(grid), dim3(256), 0, st, (const u32x4 *)a, n16, (uint32_t *)b); break;
        case ETF_PROBE_WRITE: hipLaunchKernelGGL(k_probe_write, dim3(grid), dim3(256), 0, st, (u32x4 *)a, n16); break;
        case ETF_PROBE_COPY: hipLaunchKernelGGL(k_probe_copy, dim3(grid), dim3(256), 0, st, (const u32x4 *)a, (u32x4 *)b, n16); break;
        case ETF_PROBE_ROWS: {
            // a multiplier near 0.618 nrows that shares no factor with nrows: consecutive rows land far apart
            uint64_t mult = (uint64_t)((double)nrows * 0.6180339887) | 1u;
            auto gcd = [](uint64_t x, uint64_t y) { while (y) { const uint64_t t = x % y; x = y; y = t; } return x; };
            while (gcd(mult, (uint64_t)nrows) != 1) mult += 2;
            hipLaunchKernelGGL(k_probe_rows, dim3(grid), dim3(256), 0, st, (const float *)a, nrows, mult, (uint32_t *)b);
            break;
        }
        case ETF_PROBE_LDS:
        case ETF_PROBE_LDS_SCATTER: {
            // one workgroup of 16 waves per compute unit and round, `bytes` read from LDS in total
            const int blocks = 256 * 4;
            int iters = (int)std::min<int64_t>(bytes / ((int64_t)blocks * 16 * 1024), 1 << 20);
            iters = std::max(8, iters & ~7);
            int rc = kind == ETF_PROBE_LDS ? set_lds(ctx, k_probe_lds<false>, 128 * 1024) : set_lds(ctx, k_probe_lds<true>, 128 * 1024);
            if (rc) return rc;
            if (kind == ETF_PROBE_LDS) hipLaunchKernelGGL(k_probe_lds<false>, dim3(blocks), dim3(1024), 128 * 1024, st, iters, (uint32_t *)b);
            else hipLaunchKernelGGL(k_probe_lds<true>, dim3(blocks), dim3(1024), 128 * 1024, st, iters, (uint32_t *)b);
            break;
        }
        case ETF_PROBE_VALU_F32:
        case ETF_PROBE_VALU_ADD3:
        case ETF_PROBE_VALU_PK16: {
            // `bytes` counts lane instructions here: 2048 workgroups x 256 lanes x 64 per iteration
            const int iters = (int)std::max<int64_t>(1, std::min<int64_t>(bytes / ((int64_t)2048 * 256 * 64), 1 << 24));
            if (kind == ETF_PROBE_VALU_F32) hipLaunchKernelGGL(k_probe_valu<0>, dim3(2048), dim3(256), 0, st, iters, (uint32_t *)b);
            else if (kind == ETF_PROBE_VALU_ADD3) hipLaunchKernelGGL(k_probe_valu<1>, dim3(2048), dim3(256), 0, st, iters, (uint32_t *)b);
            else hipLaunchKernelGGL(k_probe_valu<2>, dim3(2048), dim3(256), 0, st, iters, (uint32_t *)b);
            break;
        }
        case ETF_PROBE_MFMA_F32: {
            // `bytes` counts floating-point operations here: 2048 workgroups x 4 waves x 32 instructions of 4096 per iteration
            const int iters = (int)std::max<int64_t>(1, std::min<int64_t>(bytes / ((int64_t)2048 * 4 * 32 * 4096), 1 << 24));
            hipLaunchKernelGGL(k_probe_mfma, dim3(2048), dim3(256), 0, st, iters, (uint32_t *)b);
            break;
        }
        default: return fail(ctx, ETF_EINVAL, "unknown probe kind %d", kind);
    }
    LAUNCH_CHECK(ctx, "k_probe");
    return ETF_OK;
}

extern "C" int64_t etf_workspace_bytes(const etf_ctx *ctx, int64_t Q, int k, int mode)
{
    if (!ctx) return ETF_EINVAL;
    Plan P;
    int rc = make_plan(ctx, Q, k, mode, k > 0, P);
    if (rc) return rc;
    return P.total;
}

// =============================================================================================
// S1 as an entry point
// =============================================================================================
extern "C" int etf_lut_build(etf_ctx *ctx, const float *queries, int64_t Q, float *lut)
{
    int rc = need_device(ctx);
    if (rc) return rc;
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks");
    if (!ctx->dev_base) return fail(ctx, ETF_ESTATE, "codebooks not on the device: call etf_index_upload first");
    if (!queries || !lut) return fail(ctx, ETF_EINVAL, "null pointer");
    if (Q <= 0) return fail(ctx, ETF_EINVAL, "Q must be positive");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    const int64_t tiles = (Q + QT - 1) / QT;
    for (int64_t t0 = 0; t0 < tiles; t0 += 32768) {
        const int64_t nt = std::min<int64_t>(32768, tiles - t0);
        rc = launch_lut(ctx, queries, Q, t0 * QT, nt, nullptr, lut);
        if (rc) return rc;
    }
    return ETF_OK;
}

// =============================================================================================
// all-pairs ADC
// =============================================================================================
extern "C" int etf_adc(etf_ctx *ctx, const float *queries, int64_t Q, int mode, float *dist, void *ws, int64_t ws_bytes)
{
    int rc = check_ready(ctx, queries, ws);
    if (rc) return rc;
    if (!dist) return fail(ctx, ETF_EINVAL, "dist pointer is null");
    Plan P;
    rc = make_plan(ctx, Q, 0, mode, false, P);
    if (rc) return rc;
    if (ws_bytes < P.total) return fail(ctx, ETF_ENOMEM, "workspace too small: %lld < %lld", (long long)ws_bytes, (long long)P.total);
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    const HostIndex &ix = ctx->idx;
    char *w = (char *)ws;
    for (int64_t t0 = 0; t0 < P.tiles_total; t0 += P.NT) {
        const int64_t tiles = std::min<int64_t>(P.NT, P.tiles_total - t0);
        const int64_t q0 = t0 * QT;
        rc = launch_lut(ctx, queries, Q, q0, tiles, reinterpret_cast<float *>(w + P.o_lutT), nullptr);
        if (rc) return rc;
        OutArgs o;
        memset(&o, 0, sizeof o);
        o.dist = dist + q0 * ix.N;
        o.N = ix.N;
        o.nq = std::min<int64_t>(tiles * QT, Q - q0);
        if (ix.has_term) {
            // the kernels that walk the input positions add the vector's term, those that walk the entries the entry's
            const bool by_position = P.flat_lds || mode == ETF_MODE_FLAT || P.lds_path;
            o.term = reinterpret_cast<const float *>(ctx->dev_base + (by_position ? ctx->lay.pterm : ctx->lay.eterm));
        }
        const uint32_t *codes_in = reinterpret_cast<const uint32_t *>(ctx->dev_base + ctx->lay.codes);
        if (P.flat_lds) {
            rc = launch_lds<OUT_ALLPAIRS, false>(ctx, P, w, codes_in, ix.N, nullptr, 1, tiles, o, ETF_K_FLAT);
            if (rc) return rc;
        } else if (mode == ETF_MODE_FLAT) {
            rc = launch_flat<OUT_ALLPAIRS>(ctx, P, w, ix.N, nullptr, tiles, o);
            if (rc) return rc;
        } else if (P.lds_path) {
            // every distance in input order: the sums of the trees, chunk by chunk from LDS
            rc = launch_lds<OUT_ALLPAIRS, false>(ctx, P, w, codes_in, ix.N, nullptr, ix.T, tiles, o, ETF_K_LDS);
            if (rc) return rc;
        } else {
            const uint32_t *enc_of_pos = reinterpret_cast<const uint32_t *>(ctx->dev_base + ctx->lay.enc_of_pos);
            ReduceArgs r;
            if (P.ctx_path) {
                rc = launch_trees_ctx(ctx, P, w, tiles);
                if (rc) return rc;
                fill_fused_args(ctx, P, w, r);
                rc = launch_fused<OUT_ALLPAIRS>(ctx, P, w, r, ix.N, enc_of_pos, tiles, o);
            } else {
                rc = launch_trees(ctx, P, w, tiles);
                if (rc) return rc;
                fill_reduce_args(ctx, P, w, r);
                rc = launch_reduce<OUT_ALLPAIRS>(ctx, r, ix.N, enc_of_pos, tiles, o);
            }
            if (rc) return rc;
        }
    }
    return ETF_OK;
}

// =============================================================================================
// device encoder
// =============================================================================================
extern "C" int64_t etf_rotate_workspace_bytes(const etf_ctx *ctx)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->rotation.empty()) return fail(ctx, ETF_ESTATE, "no rotation: call etf_pq_set_rotation or etf_opq_train first");
    return (int64_t)((ctx->rotation.size() * sizeof(float) + 255) & ~(size_t)255);
}

extern "C" int etf_rotate_device(etf_ctx *ctx, const float *x, int64_t n, float *out, void *ws, int64_t ws_bytes)
{
    int rc = need_device(ctx);
    if (rc) return rc;
    if (ctx->rotation.empty()) return fail(ctx, ETF_ESTATE, "no rotation: call etf_pq_set_rotation or etf_opq_train first");
    if (n < 0 || (n > 0 && (!x || !out))) return fail(ctx, ETF_EINVAL, "null input or output with n=%lld", (long long)n);
    if (x == out && n > 0) return fail(ctx, ETF_EINVAL, "the rotation does not work in place");
    if (!ws || ((uintptr_t)ws & 255) != 0) return fail(ctx, ETF_EINVAL, "workspace is null or not 256-byte aligned");
    const int64_t need = etf_rotate_workspace_bytes(ctx);
    if (ws_bytes < need) return fail(ctx, ETF_ENOMEM, "workspace too small: %lld < %lld", (long long)ws_bytes, (long long)need);
    if (n == 0) return ETF_OK;
    const int d = ctx->rot_d;
    const int rows_per_block = std::max(1, std::min(8, 16384 / d));  // at most 64 KB of LDS
    if ((n + rows_per_block - 1) / rows_per_block > 0x7FFFFFFF) return fail(ctx, ETF_EINVAL, "n too large for one launch");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t st = (hipStream_t)ctx->stream;
    // the transposed rotation goes to the workspace (kept in the context so that the copy's source outlives the call)
    try {
        ctx->rotation_t.resize(ctx->rotation.size());
    } catch (const std::bad_alloc &) {
        return fail(ctx, ETF_ENOMEM, "out of host memory");
    }
    for (int r = 0; r < d; ++r)
        for (int j = 0; j < d; ++j) ctx->rotation_t[(size_t)j * d + r] = ctx->rotation[(size_t)r * d + j];
    HIP_TRY(ctx, hipMemcpyAsync(ws, ctx->rotation_t.data(), ctx->rotation_t.size() * sizeof(float), hipMemcpyHostToDevice, st));
    hipLaunchKernelGGL(k_rotate, dim3((unsigned)((n + rows_per_block - 1) / rows_per_block)), dim3(256),
                       (size_t)rows_per_block * d * sizeof(float), st, x, n, d, reinterpret_cast<const float *>(ws), out, rows_per_block);
    LAUNCH_CHECK(ctx, "k_rotate");
    return ETF_OK;
}

extern "C" int64_t etf_encode_workspace_bytes(const etf_ctx *ctx)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks: call etf_pq_train or etf_pq_set_codebooks first");
    // the codebooks, then per group 256 halved squared norms and the largest norm (k_encode_norms)
    return (int64_t)((ctx->codebooks.size() * sizeof(float) + 255) & ~(size_t)255) + (int64_t)(((size_t)ctx->M * 257 * sizeof(float) + 255) & ~(size_t)255);
}

extern "C" int etf_pq_encode_device(etf_ctx *ctx, const float *x, int64_t n, uint8_t *codes_out, void *ws, int64_t ws_bytes)
{
    int rc = need_device(ctx);
    if (rc) return rc;
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks: call etf_pq_train or etf_pq_set_codebooks first");
    if (n < 0 || (n > 0 && (!x || !codes_out))) return fail(ctx, ETF_EINVAL, "null input or output with n=%lld", (long long)n);
    if (!ws || ((uintptr_t)ws & 255) != 0) return fail(ctx, ETF_EINVAL, "workspace is null or not 256-byte aligned");
    const int64_t need = etf_encode_workspace_bytes(ctx);
    if (ws_bytes < need) return fail(ctx, ETF_ENOMEM, "workspace too small: %lld < %lld", (long long)ws_bytes, (long long)need);
    const int d = ctx->d, M = ctx->M, K = ctx->K, ds = ctx->ds;
    const bool mfma = ctx->opt.encode_kernel == 0;
    if (!mfma && ds > 128) return fail(ctx, ETF_EINVAL, "the plain device encoder handles at most 128 dimensions per group (d/M = %d)", ds);
    if (n == 0) return ETF_OK;
    if ((n + 255) / 256 > 0x7FFFFFFF) return fail(ctx, ETF_EINVAL, "n too large for one launch");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t st = (hipStream_t)ctx->stream;
    HIP_TRY(ctx, hipMemcpyAsync(ws, ctx->codebooks.data(), ctx->codebooks.size() * sizeof(float), hipMemcpyHostToDevice, st));
    const float *cb = reinterpret_cast<const float *>(ws);
    if (mfma) {
        ProfScope prof(ctx, ETF_K_ENCODE);
        const bool aligned = (ds & 3) == 0 && (d & 3) == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0;
        if (aligned && ds <= 64 && K <= 256) {
            float *cc2 = reinterpret_cast<float *>((char *)ws + ((ctx->codebooks.size() * sizeof(float) + 255) & ~(size_t)255));
            hipLaunchKernelGGL(k_encode_norms, dim3((unsigned)M), dim3(256), 0, st, cb, ds, K, M, cc2);
            // operands staged in LDS in instruction order; stretches of 128 vectors per workgroup, as many as leave
            // about eight workgroups per compute unit
            const int64_t chunks = (n + 127) / 128;
            const int reps = (int)std::max<int64_t>(1, std::min<int64_t>(16, chunks * M / 2048));
            const dim3 grid((unsigned)((chunks + reps - 1) / reps), (unsigned)M);
#define TC_CASE(RL, NB)                                                                                        \
    {                                                                                                         \
        const size_t lds = (size_t)256 * NB * 2 * RL * 4;                                                     \
        int rc2 = set_lds(ctx, k_encode_tc<RL, NB>, lds);                                                     \
        if (rc2) return rc2;                                                                                  \
        hipLaunchKernelGGL((k_encode_tc<RL, NB>), grid, dim3(256), lds, st, x, n, d, ds, K, M, cb, cc2, codes_out, reps); \
    }
            if (ds <= 8) TC_CASE(4, 1)
            else if (ds <= 16) TC_CASE(8, 1)
            else if (ds <= 32) TC_CASE(8, 2)
            else TC_CASE(8, 4)
#undef TC_CASE
            LAUNCH_CHECK(ctx, "k_encode_tc");
            return ETF_OK;
        }
        if (aligned && ds > 64 && K <= 256 && (int64_t)127 * d < ((int64_t)1 << 31) && ctx->opt.encode_wide != 0) {
            // wide groups: both operands through LDS
            float *cc2 = reinterpret_cast<float *>((char *)ws + ((ctx->codebooks.size() * sizeof(float) + 255) & ~(size_t)255));
            hipLaunchKernelGGL(k_encode_norms, dim3((unsigned)M), dim3(256), 0, st, cb, ds, K, M, cc2);
            hipLaunchKernelGGL(k_encode_wide, dim3((unsigned)((n + 127) / 128), (unsigned)M), dim3(256), 0, st, x, n, d, ds, K, M, cb, cc2, codes_out);
            LAUNCH_CHECK(ctx, "k_encode_wide");
            return ETF_OK;
        }
        hipLaunchKernelGGL(k_encode_mfma, dim3((unsigned)((n + 255) / 256), (unsigned)M), dim3(256), 0, st, x, n, d, ds, K, M, cb, codes_out);
        LAUNCH_CHECK(ctx, "k_encode_mfma");
        return ETF_OK;
    }
    int dsp = 4;
    while (dsp < ds) dsp <<= 1;
    const int KC = (int)std::min<int64_t>(K, LDS_BUDGET / (dsp * 4));
    const size_t lds = (size_t)KC * dsp * 4;
    dim3 grid((unsigned)((n + 255) / 256), (unsigned)M);
    ProfScope prof(ctx, ETF_K_ENCODE);
#define ENC_CASE(DSP)                                                                                     \
    case DSP: {                                                                                           \
        int rc2 = set_lds(ctx, k_encode<DSP>, lds);                                                       \
        if (rc2) return rc2;                                                                              \
        hipLaunchKernelGGL(k_encode<DSP>, grid, dim3(256), lds, st, x, n, d, ds, K, M, cb, codes_out, KC); \
        break;                                                                                            \
    }
    switch (dsp) {
        ENC_CASE(4)
        ENC_CASE(8)
        ENC_CASE(16)
        ENC_CASE(32)
        ENC_CASE(64)
        ENC_CASE(128)
        default: return fail(ctx, ETF_EINVAL, "no encoder for %d dimensions per group", ds);
    }
#undef ENC_CASE
    LAUNCH_CHECK(ctx, "k_encode");
    return ETF_OK;
}

// =============================================================================================
// top-k search
// =============================================================================================
// ws_cap > 0: the workspace is the fixed scratch array of the allocation-free entry point
static int search_impl(etf_ctx *ctx, const float *queries, int64_t Q, int k, int mode, int32_t *out_ids, float *out_dist,
                       void *ws, int64_t ws_bytes, int64_t ws_cap)
{
    int rc = check_ready(ctx, queries, ws);
    if (rc) return rc;
    if (!out_ids || !out_dist) return fail(ctx, ETF_EINVAL, "output pointer is null");
    Plan P;
    rc = make_plan(ctx, Q, k, mode, true, P, ws_cap);
    if (rc) return rc;
    if (ws_bytes < P.total) {
        if (ws_cap > 0)
            return fail(ctx, ETF_ENOMEM, "this search needs %lld bytes of scratch for one tile of 64 queries; the allocation-free entry point has %lld",
                        (long long)P.total, (long long)ws_bytes);
        return fail(ctx, ETF_ENOMEM, "workspace too small: %lld < %lld", (long long)ws_bytes, (long long)P.total);
    }
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t st = (hipStream_t)ctx->stream;
    const HostIndex &ix = ctx->idx;
    const DevLayout &L = ctx->lay;
    char *w = (char *)ws;
    const bool flat = mode == ETF_MODE_FLAT;
    uint32_t *counter = reinterpret_cast<uint32_t *>(w + P.o_counter);
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, counter, (int64_t)64, 0u);
    LAUNCH_CHECK(ctx, "k_fill_u32");
    ctx->last_flag_count = counter;
    for (int64_t t0 = 0; t0 < P.tiles_total; t0 += P.NT) {
        const int64_t tiles = std::min<int64_t>(P.NT, P.tiles_total - t0);
        const int64_t q0 = t0 * QT;
        const int64_t nq = std::min<int64_t>(tiles * QT, Q - q0);
        const int64_t nql = tiles * QT;
        float *lutT = reinterpret_cast<float *>(w + P.o_lutT);
        float *tau = reinterpret_cast<float *>(w + P.o_tau);
        uint32_t *cnt = reinterpret_cast<uint32_t *>(w + P.o_cnt);
        uint32_t *flag = reinterpret_cast<uint32_t *>(w + P.o_flag);
        uint64_t *cand = reinterpret_cast<uint64_t *>(w + P.o_cand);
        rc = launch_lut(ctx, queries, Q, q0, tiles, lutT, nullptr);
        if (rc) return rc;
        float *boff = nullptr;
        if (ctx->opt.metric == 1) {  // the selection orders non-negative values, smallest first
            boff = reinterpret_cast<float *>(w + P.o_boff);
            ProfScope prof(ctx, ETF_K_LUT);
            float *bm = reinterpret_cast<float *>(w + P.o_bm);
            hipLaunchKernelGGL(k_lut_shift, dim3((unsigned)tiles, (unsigned)ix.M), dim3(256), 0, st, lutT, ix.M, ix.K, bm);
            LAUNCH_CHECK(ctx, "k_lut_shift");
            hipLaunchKernelGGL(k_lut_shift_sum, dim3((unsigned)tiles), dim3(64), 0, st, bm, ix.M, boff);
            LAUNCH_CHECK(ctx, "k_lut_shift_sum");
        }
        const unsigned fb = (unsigned)((nql + 255) / 256);
        hipLaunchKernelGGL(k_fill_u32, dim3(fb), dim3(256), 0, st, cnt, nql, 0u);
        hipLaunchKernelGGL(k_fill_u32, dim3(fb), dim3(256), 0, st, flag, nql, ctx->opt.force_fallback ? 1u : 0u);
        LAUNCH_CHECK(ctx, "k_fill_u32");
        OutArgs o;
        memset(&o, 0, sizeof o);
        o.gmin = P.use_tau ? reinterpret_cast<float *>(w + P.o_gmin) : nullptr;
        o.ngroups = P.ngroups;
        o.gsize = P.gsize;
        o.tau = tau;
        o.cnt = cnt;
        o.cand = cand;
        o.C = P.C;
        o.nq = nq;
        const float *term = nullptr;
        if (ix.has_term) {
            term = reinterpret_cast<const float *>(ctx->dev_base + (flat ? L.pterm : L.eterm));
            o.term = term;
            o.term_map = reinterpret_cast<const uint32_t *>(ctx->dev_base + (flat ? L.sample_pos : L.sample_enc));
        }
        ReduceArgs r;
        const uint32_t *ecodes = reinterpret_cast<const uint32_t *>(ctx->dev_base + L.ecodes);
        if (!flat && !P.lds_path) {
            rc = P.ctx_path ? launch_trees_ctx(ctx, P, w, tiles) : launch_trees(ctx, P, w, tiles);
            if (rc) return rc;
            if (P.ctx_path) fill_fused_args(ctx, P, w, r);
            else fill_reduce_args(ctx, P, w, r);
        }
        if (!ctx->opt.force_fallback) {
            if (P.use_tau) {
                if (flat)
                    rc = launch_flat<OUT_SAMPLE>(ctx, P, w, P.S, reinterpret_cast<const uint32_t *>(ctx->dev_base + L.sample_pos), tiles, o);
                else if (P.lds_path)
                    rc = launch_lds<OUT_SAMPLE, false>(ctx, P, w, reinterpret_cast<const uint32_t *>(ctx->dev_base + L.sample_enc_codes), P.S,
                                                       nullptr, ix.T, tiles, o, ETF_K_SAMPLE);
                else
                    rc = P.ctx_path ? launch_fused<OUT_SAMPLE>(ctx, P, w, r, P.S, reinterpret_cast<const uint32_t *>(ctx->dev_base + L.sample_enc), tiles, o)
                                    : launch_reduce<OUT_SAMPLE>(ctx, r, P.S, reinterpret_cast<const uint32_t *>(ctx->dev_base + L.sample_enc), tiles, o);
                if (rc) return rc;
                {
                    ProfScope prof(ctx, ETF_K_TAU);
                    // three digits: the bound is the top of a bucket 2^-16 of its value wide (the fourth pass bought nothing)
                    hipLaunchKernelGGL(k_tau, dim3((unsigned)tiles), dim3(1024), 0, st, o.gmin, P.ngroups, k, 3, nq, tau);
                }
                LAUNCH_CHECK(ctx, "k_tau");
            } else {
                hipLaunchKernelGGL(k_fill_f32, dim3(fb), dim3(256), 0, st, tau, nql, nq, __builtin_inff(), -1.f);
                LAUNCH_CHECK(ctx, "k_fill_f32");
            }
            if (flat)
                rc = launch_flat<OUT_FILTER>(ctx, P, w, ix.N, nullptr, tiles, o);
            else if (P.lds_path)
                rc = P.fx16 ? launch_lds16(ctx, P, w, ecodes, ix.Nd, tiles, o)
                    : P.fx ? launch_lds<OUT_FILTER, true, true>(ctx, P, w, ecodes, ix.Nd, nullptr, ix.T, tiles, o, ETF_K_LDS)
                    : ix.has_term ? launch_lds<OUT_FILTER, true, false, true>(ctx, P, w, ecodes, ix.Nd, nullptr, ix.T, tiles, o, ETF_K_LDS)
                                  : launch_lds<OUT_FILTER, true>(ctx, P, w, ecodes, ix.Nd, nullptr, ix.T, tiles, o, ETF_K_LDS);
            else
                rc = P.ctx_path ? launch_fused<OUT_FILTER>(ctx, P, w, r, ix.Nd, nullptr, tiles, o)
                                : launch_reduce<OUT_FILTER>(ctx, r, ix.Nd, nullptr, tiles, o);
            if (rc) return rc;
        }
        SelectArgs sa;
        memset(&sa, 0, sizeof sa);
        sa.cnt = cnt;
        sa.cand = cand;
        sa.C = P.C;
        sa.ebegin = flat ? nullptr : reinterpret_cast<const uint32_t *>(ctx->dev_base + L.ebegin);
        sa.ids = reinterpret_cast<const int32_t *>(ctx->dev_base + (flat ? L.ids_in : L.ids_sorted));
        sa.k = k;
        sa.out_ids = out_ids + q0 * k;
        sa.out_dist = out_dist + q0 * k;
        sa.flag = flag;
        sa.boff = boff;
        // fixed-point candidates: rounding moves a sum by at most M units (truncated entries) plus 2^-24 relative per
        // entry and per float32 addition of the distance it stands for, 2^27 * (M + 1) * 2^-24 = 8 (M + 1) units at the
        // bound; twice that between two candidates
        sa.fx_margin = P.fx ? (uint32_t)(2 * (ix.M + 8 * (ix.M + 1)) + 16) : 0u;
        // 16-bit tables: truncation makes a sum too small by at most M units, everything else is far below one unit
        if (P.fx16) sa.fx_margin = (uint32_t)(ix.M + 2);
        sa.fx_first_pass = P.fx16 ? 2 : 0;
        sa.lutT = lutT;
        sa.codes = reinterpret_cast<const uint8_t *>(ctx->dev_base + (flat ? L.codes : L.ecodes));
        sa.term = term;
        sa.M = ix.M;
        sa.K = ix.K;
        sa.grouped = (P.lds_path || P.flat_lds) ? lds_chunks_per_line(std::max(2, pick_G(ix.M, ix.K))) : 0;
        sa.T = flat ? 1 : ix.T;
        for (int t = 0; t <= ETF_MAX_M; ++t) sa.chunk_begin[t] = 0;
        if (flat) sa.chunk_begin[1] = ix.M;
        else for (int t = 0; t <= ix.T; ++t) sa.chunk_begin[t] = ix.chunk_begin[t];
        {
            ProfScope prof(ctx, ETF_K_SELECT);
            hipLaunchKernelGGL(k_select, dim3((unsigned)nq), dim3(256), select_lds_bytes(k), st, sa);
        }
        LAUNCH_CHECK(ctx, "k_select");
        ExactArgs ea;
        memset(&ea, 0, sizeof ea);
        ea.flag = flag;
        ea.nflag = counter;
        ea.lutT = lutT;
        ea.M = ix.M;
        ea.K = ix.K;
        ea.grouped = (P.lds_path || P.flat_lds) ? lds_chunks_per_line(std::max(2, pick_G(ix.M, ix.K))) : 0;
        if (flat) {
            ea.T = 1;
            ea.chunk_begin[0] = 0;
            ea.chunk_begin[1] = ix.M;
            ea.codes = reinterpret_cast<const uint8_t *>(ctx->dev_base + L.codes);
            ea.rows = ix.N;
            ea.ebegin = nullptr;
        } else {
            ea.T = ix.T;
            for (int t = 0; t <= ix.T; ++t) ea.chunk_begin[t] = ix.chunk_begin[t];
            ea.codes = reinterpret_cast<const uint8_t *>(ctx->dev_base + L.ecodes);
            ea.rows = ix.Nd;
            ea.ebegin = sa.ebegin;
        }
        ea.term = term;
        ea.ids = sa.ids;
        ea.k = k;
        ea.out_ids = sa.out_ids;
        ea.out_dist = sa.out_dist;
        ea.boff = boff;
        {
            ProfScope prof(ctx, ETF_K_EXACT);
            hipLaunchKernelGGL(k_exact, dim3((unsigned)nq), dim3(256), 0, st, ea);
        }
        LAUNCH_CHECK(ctx, "k_exact");
    }
    return ETF_OK;
}

extern "C" int etf_search(etf_ctx *ctx, const float *queries, int64_t Q, int k, int mode, int32_t *out_ids,
                          float *out_dist, void *ws, int64_t ws_bytes)
{
    return search_impl(ctx, queries, Q, k, mode, out_ids, out_dist, ws, ws_bytes, 0);
}

// =============================================================================================
// the search without any allocation
// =============================================================================================
// Scratch of etf_search_static: one array per GPU the library runs on, held until the process ends and shared by
// every call on that GPU.  In host code the array's name is only a handle for hipGetSymbolAddress; the address
// kernels and copies use is looked up once per device (etf_create) and kept in g_scratch.
static __device__ __align__(256) unsigned char scratch[ETF_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void *g_scratch[MAX_DEVICES];          // device address of `scratch` on every device seen so far
hipError_t g_scratch_err[MAX_DEVICES];
bool g_scratch_tried[MAX_DEVICES];
std::mutex g_scratch_mu;
}  // namespace

// called by etf_create with a device context; the device is made current here
static void lookup_scratch(int device)
{
    if (device < 0 || device >= MAX_DEVICES) return;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_tried[device]) return;
    g_scratch_tried[device] = true;
    hipError_t e = hipSetDevice(device);
    void *p = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    g_scratch_err[device] = e;
    g_scratch[device] = e == hipSuccess ? p : nullptr;
}

extern "C" int64_t etf_static_scratch_bytes(void) { return (int64_t)ETF_STATIC_SCRATCH_BYTES; }

extern "C" int etf_search_static(etf_ctx *ctx, const float *queries, int64_t Q, int k, int mode, int32_t *out_ids,
                                 float *out_dist)
{
    int rc = need_device(ctx);
    if (rc) return rc;
    if (ctx->device >= MAX_DEVICES) return fail(ctx, ETF_EINVAL, "device %d: the scratch table holds %d devices", ctx->device, MAX_DEVICES);
    void *ws;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        ws = g_scratch[ctx->device];
        if (!ws)
            return fail(ctx, ETF_EHIP, "the scratch array has no address on device %d: %s", ctx->device,
                        g_scratch_tried[ctx->device] ? hipGetErrorString(g_scratch_err[ctx->device]) : "etf_create did not look it up");
    }
    ctx->no_alloc_call = true;  // no event pairs around the launches: creating an event allocates
    rc = search_impl(ctx, queries, Q, k, mode, out_ids, out_dist, ws, ETF_STATIC_SCRATCH_BYTES, ETF_STATIC_SCRATCH_BYTES);
    ctx->no_alloc_call = false;
    return rc;
}

extern "C" int etf_last_fallback_count(etf_ctx *ctx, int64_t *out)
{
    int rc = need_device(ctx);
    if (rc) return rc;
    if (!out) return fail(ctx, ETF_EINVAL, "output pointer is null");
    if (!ctx->last_flag_count) return fail(ctx, ETF_ESTATE, "no search has run on this context");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, hipStreamSynchronize((hipStream_t)ctx->stream));
    uint32_t v = 0;
    HIP_TRY(ctx, hipMemcpy(&v, ctx->last_flag_count, sizeof v, hipMemcpyDeviceToHost));
    *out = v;
    return ETF_OK;
}

#include "etf_ivf.hip.h"
