// Host half of the library: context, product quantiser (train / encode), index build, statistics.
//
// The index build follows the paper's "Constructing Encoding Tree": sort the encodings
// lexicographically, then grow the tree in one linear, append-only pass driven by the longest
// common prefix of neighbouring encodings (Algorithm 1).  What differs from the paper is the
// serialisation: instead of one depth-first byte stream (Hierarchical Memory Structure) the nodes
// are appended to one array per level.  Because the input is sorted, each of these arrays is in
// breadth-first order, the children of a node are adjacent, and the leaves in sorted order are the
// paper's depth-first leaf order.
#include <algorithm>
#include <atomic>
#include <cfloat>
#include <cmath>
#include <cstdarg>
#include <cstring>
#include <functional>
#include <thread>

#include "etf_internal.h"

namespace etf {

int fail(const etf_ctx *ctx, int code, const char *fmt, ...)
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

int host_threads()
{
    unsigned hc = std::thread::hardware_concurrency();
    int t = hc ? (int)hc : 4;
    if (const char *e = getenv("OMP_NUM_THREADS")) {
        int v = atoi(e);
        if (v > 0) t = std::min(t, v);
    }
    return std::max(1, std::min(t, 64));
}

void parallel_slices(int64_t n, int threads, const std::function<void(int, int64_t, int64_t)> &fn)
{
    if (n <= 0) return;
    threads = (int)std::max<int64_t>(1, std::min<int64_t>(threads, n));
    if (threads == 1) {
        fn(0, 0, n);
        return;
    }
    std::vector<std::thread> th;
    th.reserve(threads);
    for (int t = 0; t < threads; ++t) {
        int64_t b = n * t / threads, e = n * (t + 1) / threads;
        th.emplace_back([&fn, t, b, e] { fn(t, b, e); });
    }
    for (auto &x : th) x.join();
}

// splitmix64: the library's own seeded generator (initial codewords, threshold sample)
static inline uint64_t splitmix64(uint64_t &s)
{
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// ---------------------------------------------------------------------------------------------
// Stable LSD radix sort of fixed-size records by a list of key bytes (least significant first).
// ---------------------------------------------------------------------------------------------
template <class Rec, class ByteOf>
static void radix_sort_records(std::vector<Rec> &a, int nbytes, ByteOf byte_of)
{
    const int64_t n = (int64_t)a.size();
    if (n < 2) return;
    std::vector<Rec> b(a.size());
    Rec *src = a.data(), *dst = b.data();
    const int threads = n > (1 << 16) ? host_threads() : 1;
    std::vector<int64_t> hist((size_t)threads * 256);
    for (int p = 0; p < nbytes; ++p) {
        std::fill(hist.begin(), hist.end(), 0);
        parallel_slices(n, threads, [&](int t, int64_t lo, int64_t hi) {
            int64_t *h = hist.data() + (size_t)t * 256;
            for (int64_t i = lo; i < hi; ++i) h[byte_of(src[i], p)]++;
        });
        // a pass in which every record has the same digit moves nothing
        bool trivial = false;
        for (int v = 0; v < 256 && !trivial; ++v) {
            int64_t c = 0;
            for (int t = 0; t < threads; ++t) c += hist[(size_t)t * 256 + v];
            if (c == n) trivial = true;
        }
        if (trivial) continue;
        int64_t run = 0;
        for (int v = 0; v < 256; ++v)
            for (int t = 0; t < threads; ++t) {
                int64_t c = hist[(size_t)t * 256 + v];
                hist[(size_t)t * 256 + v] = run;
                run += c;
            }
        parallel_slices(n, threads, [&](int t, int64_t lo, int64_t hi) {
            int64_t *h = hist.data() + (size_t)t * 256;
            for (int64_t i = lo; i < hi; ++i) dst[h[byte_of(src[i], p)]++] = src[i];
        });
        std::swap(src, dst);
    }
    if (src != a.data()) a.swap(b);
}

struct KeyRec {
    uint64_t k[2];   // code bytes packed big-endian: integer order == lexicographic order
    uint32_t pos;    // payload: input position or distinct-encoding number
    int32_t id;      // last key
    uint32_t tb;     // bits of the vector's leaf term (non-negative float: orders like the value), 0 without payload
};

static inline void pack_key(const uint8_t *code, int c0, int c1, uint64_t k[2])
{
    k[0] = k[1] = 0;
    for (int m = c0; m < c1; ++m) {
        int j = m - c0;
        k[j >> 3] |= (uint64_t)code[m] << (56 - 8 * (j & 7));
    }
}

static inline int key_byte(const uint64_t k[2], int j) { return (int)((k[j >> 3] >> (56 - 8 * (j & 7))) & 255); }

// longest common prefix, in chunks, of two packed keys of D chunks
static inline int key_lcp(const uint64_t a[2], const uint64_t b[2], int D)
{
    for (int w = 0; w < 2; ++w) {
        uint64_t x = a[w] ^ b[w];
        if (x) return std::min(D, w * 8 + (__builtin_clzll(x) >> 3));
    }
    return D;
}

// ---------------------------------------------------------------------------------------------
// One tree over sorted distinct sub-encodings (Algorithm 1, level-ordered output).
// ---------------------------------------------------------------------------------------------
static void build_tree(const std::vector<KeyRec> &sub /* sorted, distinct keys */, int D, HostTree &tr)
{
    const int64_t U = (int64_t)sub.size();
    tr.U = U;
    tr.level.assign(D, HostLevel());
    tr.bucket.assign(D, HostBucket());
    for (int l = 0; l < D; ++l) {
        tr.bucket[l].width = D - l;                       // own chunk + postfix of D-(l+1)
        tr.bucket[l].stride = (tr.bucket[l].width + 3) & ~3;
    }
    // cur[l] = internal node of level l (1-based) that the current path runs through, or NO_PARENT
    uint32_t cur[ETF_MAX_M + 1];
    for (int l = 0; l <= D; ++l) cur[l] = NO_PARENT;
    int lcp_prev = 0;  // common prefix with the previous encoding
    for (int64_t i = 0; i < U; ++i) {
        const int lcp_next = (i + 1 < U) ? key_lcp(sub[i].k, sub[i + 1].k, D) : 0;
        // the path diverges from the previous one after lcp_prev chunks: every level below that starts
        // a new prefix group; it is an internal node iff the next encoding still shares it
        for (int l = lcp_prev + 1; l <= D - 1; ++l) {
            if (lcp_next >= l) {
                HostLevel &L = tr.level[l - 1];
                L.code.push_back((uint8_t)key_byte(sub[i].k, l - 1));
                L.parent.push_back(l > 1 ? cur[l - 1] : NO_PARENT);
                cur[l] = (uint32_t)(L.code.size() - 1);
            } else {
                cur[l] = NO_PARENT;
            }
        }
        // the first level at which this encoding is alone in its prefix group: its leaf
        const int lev = 1 + std::max(lcp_prev, lcp_next);
        HostBucket &B = tr.bucket[lev - 1];
        const size_t at = B.codes.size();
        B.codes.resize(at + B.stride, 0);
        for (int j = 0; j < B.width; ++j) B.codes[at + j] = (uint8_t)key_byte(sub[i].k, lev - 1 + j);
        B.parent.push_back(lev > 1 ? cur[lev - 1] : NO_PARENT);
        B.row.push_back((uint32_t)i);
        lcp_prev = lcp_next;
    }
    tr.nI.resize(D);
    tr.nL.resize(D);
    for (int l = 0; l < D; ++l) {
        tr.nI[l] = (int64_t)tr.level[l].code.size();
        tr.nL[l] = (int64_t)tr.bucket[l].size();
    }
    // the same leaves as plain padded records in lexicographic order (register-context traversal)
    // (padded at the front to the unrolled depth, so that the deepest level is always the last slot)
    tr.rstride = std::max(4, depth_class(D));
    tr.rec.assign((size_t)U * tr.rstride, 0);
    const int pad = depth_class(D) - D;
    for (int64_t i = 0; i < U; ++i)
        for (int j = 0; j < D; ++j) tr.rec[(size_t)i * tr.rstride + pad + j] = (uint8_t)key_byte(sub[i].k, j);
}

static int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

// Operands of the matrix-core table build.  ||q - c||^2 = ||q'||^2 - 2 q'.c' + ||c'||^2 holds for any common
// shift q' = q - mu, c' = c - mu; the group's mean codeword as mu keeps the three terms small, so the
// cancellation in float32 stays well inside the distance tolerance.  Norms are summed in double.
void prepare_centered(etf_ctx *ctx)
{
    const int M = ctx->M, K = ctx->K, ds = ctx->ds;
    ctx->dsp = (ds + 1) & ~1;
    ctx->cb_mean.assign((size_t)M * ds, 0.f);
    ctx->cb_centered.assign((size_t)M * K * ctx->dsp, 0.f);
    ctx->cb_norm.assign((size_t)M * K, 0.f);
    for (int m = 0; m < M; ++m) {
        for (int j = 0; j < ds; ++j) {
            double s = 0.0;
            for (int k = 0; k < K; ++k) s += ctx->codebooks[((size_t)m * K + k) * ds + j];
            ctx->cb_mean[(size_t)m * ds + j] = (float)(s / K);
        }
        for (int k = 0; k < K; ++k) {
            double nn = 0.0;
            for (int j = 0; j < ds; ++j) {
                const float c = ctx->codebooks[((size_t)m * K + k) * ds + j] - ctx->cb_mean[(size_t)m * ds + j];
                ctx->cb_centered[((size_t)m * K + k) * ctx->dsp + j] = c;
                nn += (double)c * (double)c;
            }
            ctx->cb_norm[(size_t)m * K + k] = (float)nn;
        }
    }
}

int64_t sample_size(const Options &opt, int64_t n)
{
    return std::max<int64_t>(opt.sample_min, (int64_t)((double)opt.sample_scale * std::sqrt((double)n)));
}

// Every array at its largest: as many distinct encodings as vectors, every tree with as many leaves, every
// internal level with half as many nodes (an internal node has at least two encodings below it).
int64_t image_bytes_bound(const etf_ctx *ctx, int64_t N, int T, const int32_t *chunk_begin)
{
    const int M = ctx->M;
    const int64_t S = std::min(N, sample_size(ctx->opt, N));
    int64_t tot = 0;
    auto take = [&](int64_t bytes) { tot = align256(tot + std::max<int64_t>(bytes, 4)); };
    take((int64_t)ctx->codebooks.size() * 4);
    take((int64_t)ctx->cb_centered.size() * 4);
    take((int64_t)ctx->cb_norm.size() * 4);
    take((int64_t)ctx->cb_mean.size() * 4);
    take(N * M); take(N * 4); take(N * 4); take((N + 1) * 4); take(N * 4); take(N * M);
    take(S * 4); take(S * 4); take(S * M); take(S * M);
    take(N * std::max(4, depth_class(chunk_begin[1] - chunk_begin[0])));
    for (int t = 0; t < T; ++t) {
        const int D = chunk_begin[t + 1] - chunk_begin[t];
        if (T > 1) take(N * 4);
        take(N * std::max(4, depth_class(D)));
        for (int l = 0; l < D; ++l) {
            take(l + 1 < D ? N / 2 : 0);
            take(l + 1 < D ? N / 2 * 4 : 0);
        }
        // the leaves of all levels together are N; every level's arrays may round up to the next 256 bytes
        tot += N * ((D + 3) & ~3) + N * 4 + N * 4 + (int64_t)D * 3 * 256;
    }
    return tot;
}

void compute_layout(etf_ctx *ctx)
{
    const HostIndex &ix = ctx->idx;
    DevLayout &L = ctx->lay;
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        int64_t o = off;
        off = align256(off + std::max<int64_t>(bytes, 4));
        return o;
    };
    L.codebooks = take((int64_t)ctx->codebooks.size() * 4);
    L.cb_centered = take((int64_t)ctx->cb_centered.size() * 4);
    L.cb_norm = take((int64_t)ctx->cb_norm.size() * 4);
    L.cb_mean = take((int64_t)ctx->cb_mean.size() * 4);
    const int M = ix.M;
    L.codes = take(ix.N * M);
    L.ids_in = take(ix.N * 4);
    L.ids_sorted = take(ix.N * 4);
    L.ebegin = take((ix.Nd + 1) * 4);
    L.enc_of_pos = take(ix.N * 4);
    L.ecodes = take(ix.Nd * M);
    L.sample_enc = take(ix.n_sample_enc * 4);
    L.sample_pos = take(ix.n_sample_pos * 4);
    L.sample_enc_codes = take(ix.n_sample_enc * M);
    L.sample_pos_codes = take(ix.n_sample_pos * M);
    L.rec0 = take(ix.Nd * ix.rstride0);
    L.tree.assign(ix.T, DevTreeLayout());
    for (int t = 0; t < ix.T; ++t) {
        const HostTree &tr = ix.tree[t];
        DevTreeLayout &TL = L.tree[t];
        TL.leaf_of = (ix.T == 1 && !ix.has_term) ? -1 : take(ix.Nd * 4);
        TL.rec = take(tr.U * tr.rstride);
        for (int l = 0; l < tr.D; ++l) {
            TL.icode[l] = take(tr.nI[l]);
            TL.iparent[l] = take(tr.nI[l] * 4);
            TL.lcodes[l] = take(tr.nL[l] * tr.bucket[l].stride);
            TL.lparent[l] = take(tr.nL[l] * 4);
            TL.lrow[l] = take(tr.nL[l] * 4);
        }
    }
    L.eterm = ix.has_term ? take(ix.Nd * 4) : -1;
    L.pterm = ix.has_term ? take(ix.N * 4) : -1;
    L.total = off;
}

void for_each_image_array(const etf_ctx *ctx, const std::function<void(int64_t, const void *, size_t)> &put)
{
    const HostIndex &ix = ctx->idx;
    const DevLayout &L = ctx->lay;
    put(L.codebooks, ctx->codebooks.data(), ctx->codebooks.size() * 4);
    put(L.cb_centered, ctx->cb_centered.data(), ctx->cb_centered.size() * 4);
    put(L.cb_norm, ctx->cb_norm.data(), ctx->cb_norm.size() * 4);
    put(L.cb_mean, ctx->cb_mean.data(), ctx->cb_mean.size() * 4);
    put(L.codes, ix.codes.data(), ix.codes.size());
    put(L.ids_in, ix.ids_in.data(), ix.ids_in.size() * 4);
    put(L.ids_sorted, ix.ids_sorted.data(), ix.ids_sorted.size() * 4);
    put(L.ebegin, ix.ebegin.data(), ix.ebegin.size() * 4);
    put(L.enc_of_pos, ix.enc_of_pos.data(), ix.enc_of_pos.size() * 4);
    put(L.ecodes, ix.ecodes.data(), ix.ecodes.size());
    put(L.sample_enc, ix.sample_enc.data(), ix.sample_enc.size() * 4);
    put(L.sample_pos, ix.sample_pos.data(), ix.sample_pos.size() * 4);
    put(L.sample_enc_codes, ix.sample_enc_codes.data(), ix.sample_enc_codes.size());
    put(L.sample_pos_codes, ix.sample_pos_codes.data(), ix.sample_pos_codes.size());
    put(L.rec0, ix.rec0.data(), ix.rec0.size());
    for (int t = 0; t < ix.T; ++t) {
        const HostTree &tr = ix.tree[t];
        const DevTreeLayout &TL = L.tree[t];
        if (TL.leaf_of >= 0) put(TL.leaf_of, tr.leaf_of.data(), tr.leaf_of.size() * 4);
        put(TL.rec, tr.rec.data(), tr.rec.size());
        for (int l = 0; l < tr.D; ++l) {
            put(TL.icode[l], tr.level[l].code.data(), tr.level[l].code.size());
            put(TL.iparent[l], tr.level[l].parent.data(), tr.level[l].parent.size() * 4);
            put(TL.lcodes[l], tr.bucket[l].codes.data(), tr.bucket[l].codes.size());
            put(TL.lparent[l], tr.bucket[l].parent.data(), tr.bucket[l].parent.size() * 4);
            put(TL.lrow[l], tr.bucket[l].row.data(), tr.bucket[l].row.size() * 4);
        }
    }
    if (L.eterm >= 0) put(L.eterm, ix.eterm.data(), ix.eterm.size() * 4);
    if (L.pterm >= 0) put(L.pterm, ix.pterm.data(), ix.pterm.size() * 4);
}

}  // namespace etf

using namespace etf;

// =============================================================================================
// context
// =============================================================================================
extern "C" const char *etf_strerror(int code)
{
    switch (code) {
        case ETF_OK: return "ok";
        case ETF_EINVAL: return "invalid argument";
        case ETF_ESTATE: return "call not valid in this state";
        case ETF_ENOMEM: return "out of memory or buffer too small";
        case ETF_EHIP: return "HIP runtime error";
        case ETF_ENOGPU: return "context has no device";
        default: return "unknown error code";
    }
}

extern "C" const char *etf_last_error(const etf_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

extern "C" int etf_set_option(etf_ctx *ctx, const char *name, int64_t value)
{
    if (!ctx || !name) return ETF_EINVAL;
    std::string n(name);
    if (n == "ws_cap_bytes") {
        if (value < ((int64_t)1 << 20)) return fail(ctx, ETF_EINVAL, "ws_cap_bytes must be at least 1 MiB");
        ctx->opt.ws_cap_bytes = value;
    } else if (n == "force_fallback") {
        if (value != 0 && value != 1) return fail(ctx, ETF_EINVAL, "force_fallback must be 0 or 1");
        ctx->opt.force_fallback = value;
    } else if (n == "sample_min") {
        if (value < 1) return fail(ctx, ETF_EINVAL, "sample_min must be positive");
        ctx->opt.sample_min = value;
    } else if (n == "sample_scale") {
        if (value < 0) return fail(ctx, ETF_EINVAL, "sample_scale must not be negative");
        ctx->opt.sample_scale = value;
    } else if (n == "traversal") {
        if (value < 0 || value > 2)
            return fail(ctx, ETF_EINVAL, "traversal must be 0 (register context), 1 (level-synchronous) or 2 (tables in LDS)");
        ctx->opt.traversal = value;
    } else if (n == "lut_kernel") {
        if (value != 0 && value != 1) return fail(ctx, ETF_EINVAL, "lut_kernel must be 0 (matrix cores) or 1 (plain sums)");
        ctx->opt.lut_kernel = value;
    } else if (n == "ivf_coarse_kernel") {
        if (value != 0 && value != 1) return fail(ctx, ETF_EINVAL, "ivf_coarse_kernel must be 0 (matrix cores) or 1 (the float32 rule for every cell)");
        ctx->opt.ivf_coarse_kernel = value;
    } else if (n == "lut_narrow_below") {
        if (value < 0) return fail(ctx, ETF_EINVAL, "lut_narrow_below must be >= 0");
        ctx->opt.lut_narrow_below = value;
    } else if (n == "encode_wide") {
        if (value != 0 && value != 1) return fail(ctx, ETF_EINVAL, "encode_wide is 0 or 1");
        ctx->opt.encode_wide = value;
    } else if (n == "ivf_coarse_tile") {
        if (value != 0 && value != 1) return fail(ctx, ETF_EINVAL, "ivf_coarse_tile is 0 or 1");
        ctx->opt.ivf_coarse_tile = value;
    } else if (n == "ivf_bound_factor") {
        if (value < 0 || value > 1000000) return fail(ctx, ETF_EINVAL, "ivf_bound_factor must be in [0, 1e6]");
        ctx->opt.ivf_bound_factor = value;
    } else if (n == "ivf_probe_slack") {
        if (value < 1 || value > 1000000000) return fail(ctx, ETF_EINVAL, "ivf_probe_slack must be in [1, 1e9]");
        ctx->opt.ivf_probe_slack = value;
    } else if (n == "ivf_probe_cap") {
        if (value < 0 || value > 8192) return fail(ctx, ETF_EINVAL, "ivf_probe_cap must be in [0, 8192]");
        ctx->opt.ivf_probe_cap = value;
    } else if (n == "lds16_context") {
        if (value < 0 || value > 1) return fail(ctx, ETF_EINVAL, "lds16_context is 0 or 1");
        ctx->opt.lds16_context = (int)value;
    } else if (n == "lds_blocks") {
        if (value < 0 || value > 65535) return fail(ctx, ETF_EINVAL, "lds_blocks out of range");
        ctx->opt.lds_blocks = value;
    } else if (n == "metric") {
        if (value != 0 && value != 1) return fail(ctx, ETF_EINVAL, "metric must be 0 (squared Euclidean distance) or 1 (scalar product)");
        ctx->opt.metric = value;
    } else if (n == "encode_kernel") {
        if (value != 0 && value != 1) return fail(ctx, ETF_EINVAL, "encode_kernel must be 0 or 1");
        ctx->opt.encode_kernel = value;
    } else if (n == "lds_filter") {
        if (value < 0 || value > 2) return fail(ctx, ETF_EINVAL, "lds_filter must be 0, 1 or 2");
        ctx->opt.lds_filter = value;
    } else if (n == "cand_cap") {
        if (value < 0 || value > (1 << 20)) return fail(ctx, ETF_EINVAL, "cand_cap out of range");
        ctx->opt.cand_cap = value;
    } else {
        return fail(ctx, ETF_EINVAL, "unknown option '%s'", name);
    }
    return ETF_OK;
}

// =============================================================================================
// product quantiser (paper: Introduction / Related Work)
// =============================================================================================
static int check_pq_shape(etf_ctx *ctx, int d, int M, int K)
{
    if (d <= 0 || M <= 0 || M > ETF_MAX_M || K <= 0 || K > 256)
        return fail(ctx, ETF_EINVAL, "need d > 0, 1 <= M <= %d, 1 <= K <= 256 (got d=%d M=%d K=%d)", ETF_MAX_M, d, M, K);
    if (d % M != 0) return fail(ctx, ETF_EINVAL, "d=%d is not a multiple of M=%d", d, M);
    return ETF_OK;
}

namespace etf {
void drop_index(etf_ctx *ctx)
{
    ctx->idx = HostIndex();
    ctx->lay = DevLayout();
    ctx->dev_base = nullptr;
    ctx->last_flag_count = nullptr;  // the diagnostics of a search on the previous index
}
}  // namespace etf

// nearest codeword of one sub-vector; float32 arithmetic, direct (a-b)^2 form, lowest index on ties
static inline int nearest_codeword(const float *x, const float *cb, int K, int ds, float *best_out)
{
    int best = 0;
    float bestd = FLT_MAX;
    for (int k = 0; k < K; ++k) {
        const float *c = cb + (size_t)k * ds;
        float s = 0.f;
        for (int j = 0; j < ds; ++j) {
            float t = x[j] - c[j];
            s += t * t;
        }
        if (s < bestd) {
            bestd = s;
            best = k;
        }
    }
    if (best_out) *best_out = bestd;
    return best;
}

extern "C" int etf_pq_set_codebooks(etf_ctx *ctx, const float *cb, int d, int M, int K)
{
    if (!ctx) return ETF_EINVAL;
    if (!cb) return fail(ctx, ETF_EINVAL, "codebooks pointer is null");
    int rc = check_pq_shape(ctx, d, M, K);
    if (rc) return rc;
    drop_index(ctx);
    ctx->next_order.clear();
    ctx->d = d; ctx->M = M; ctx->K = K; ctx->ds = d / M;
    try {
        ctx->codebooks.assign(cb, cb + (size_t)M * K * ctx->ds);
        prepare_centered(ctx);
    } catch (const std::bad_alloc &) {
        return fail(ctx, ETF_ENOMEM, "out of host memory");
    }
    return ETF_OK;
}

extern "C" int etf_pq_get_codebooks(const etf_ctx *ctx, float *cb_out)
{
    if (!ctx) return ETF_EINVAL;
    if (!cb_out) return fail(ctx, ETF_EINVAL, "output pointer is null");
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks: call etf_pq_train or etf_pq_set_codebooks first");
    memcpy(cb_out, ctx->codebooks.data(), ctx->codebooks.size() * sizeof(float));
    return ETF_OK;
}

extern "C" int etf_pq_train(etf_ctx *ctx, const float *x, int64_t n, int d, int M, int K, int iters, uint64_t seed)
{
    if (!ctx) return ETF_EINVAL;
    if (!x || n <= 0) return fail(ctx, ETF_EINVAL, "training set is empty or null");
    if (iters < 0) return fail(ctx, ETF_EINVAL, "iters must be >= 0");
    int rc = check_pq_shape(ctx, d, M, K);
    if (rc) return rc;
    const int ds = d / M;
    try {
        std::vector<float> cb((size_t)M * K * ds);
        std::vector<int> assign((size_t)n);
        const int threads = host_threads();
        for (int m = 0; m < M; ++m) {
            float *c = cb.data() + (size_t)m * K * ds;
            // initial codewords: the first K rows of a seeded Fisher-Yates shuffle (with replacement if n < K)
            uint64_t s = seed * 0x9E3779B97F4A7C15ull + (uint64_t)m + 1;
            std::vector<int64_t> pick(K);
            if (n >= K) {
                std::vector<int64_t> perm((size_t)n);
                for (int64_t i = 0; i < n; ++i) perm[i] = i;
                for (int k = 0; k < K; ++k) {
                    int64_t j = k + (int64_t)(splitmix64(s) % (uint64_t)(n - k));
                    std::swap(perm[k], perm[j]);
                    pick[k] = perm[k];
                }
            } else {
                for (int k = 0; k < K; ++k) pick[k] = (int64_t)(splitmix64(s) % (uint64_t)n);
            }
            for (int k = 0; k < K; ++k)
                memcpy(c + (size_t)k * ds, x + (size_t)pick[k] * d + (size_t)m * ds, sizeof(float) * ds);
            for (int it = 0; it < iters; ++it) {
                parallel_slices(n, threads, [&](int, int64_t lo, int64_t hi) {
                    for (int64_t i = lo; i < hi; ++i)
                        assign[i] = nearest_codeword(x + (size_t)i * d + (size_t)m * ds, c, K, ds, nullptr);
                });
                std::vector<double> sum((size_t)K * ds, 0.0);
                std::vector<int64_t> cnt(K, 0);
                for (int64_t i = 0; i < n; ++i) {
                    const float *xi = x + (size_t)i * d + (size_t)m * ds;
                    double *sk = sum.data() + (size_t)assign[i] * ds;
                    cnt[assign[i]]++;
                    for (int j = 0; j < ds; ++j) sk[j] += xi[j];
                }
                for (int k = 0; k < K; ++k)
                    if (cnt[k])  // an empty cluster keeps its previous codeword
                        for (int j = 0; j < ds; ++j) c[(size_t)k * ds + j] = (float)(sum[(size_t)k * ds + j] / (double)cnt[k]);
            }
        }
        drop_index(ctx);
        ctx->next_order.clear();
        ctx->d = d; ctx->M = M; ctx->K = K; ctx->ds = ds;
        ctx->codebooks.swap(cb);
        prepare_centered(ctx);
    } catch (const std::bad_alloc &) {
        return fail(ctx, ETF_ENOMEM, "out of host memory");
    }
    return ETF_OK;
}

// ---- rotation in front of the quantiser (paper, Related Work: Optimized Product Quantization rotates the space so
//      that the dimension groups become less dependent; named in the survey of methods the tree applies to) --------
// y = R x, every component accumulated in double over the dimensions in ascending order (a product of two floats is
// exact in double, so fused or not makes no difference) and rounded to float once: the one rule host, device and
// reference follow, so that codes of rotated vectors can be compared bit for bit.
static void rotate_rows(const float *R, int d, const float *x, int64_t lo, int64_t hi, float *out)
{
    for (int64_t i = lo; i < hi; ++i) {
        const float *xi = x + (size_t)i * d;
        for (int r = 0; r < d; ++r) {
            const float *Rr = R + (size_t)r * d;
            double acc = 0.0;
            for (int j = 0; j < d; ++j) acc += (double)Rr[j] * (double)xi[j];
            out[(size_t)i * d + r] = (float)acc;
        }
    }
}

extern "C" int etf_pq_set_rotation(etf_ctx *ctx, const float *R, int d)
{
    if (!ctx) return ETF_EINVAL;
    if (!R) {
        ctx->rotation.clear();
        ctx->rot_d = 0;
        return ETF_OK;
    }
    if (d < 1 || d > 4096) return fail(ctx, ETF_EINVAL, "rotation of %d dimensions", d);
    for (size_t i = 0; i < (size_t)d * d; ++i)
        if (!std::isfinite(R[i])) return fail(ctx, ETF_EINVAL, "the rotation has an entry that is not finite");
    try {
        ctx->rotation.assign(R, R + (size_t)d * d);
    } catch (const std::bad_alloc &) {
        return fail(ctx, ETF_ENOMEM, "out of host memory");
    }
    ctx->rot_d = d;
    return ETF_OK;
}

extern "C" int etf_pq_get_rotation(const etf_ctx *ctx, float *R_out)
{
    if (!ctx) return ETF_EINVAL;
    if (!R_out) return fail(ctx, ETF_EINVAL, "output pointer is null");
    if (ctx->rotation.empty()) return fail(ctx, ETF_ESTATE, "no rotation: call etf_pq_set_rotation or etf_opq_train first");
    memcpy(R_out, ctx->rotation.data(), ctx->rotation.size() * sizeof(float));
    return ETF_OK;
}

extern "C" int etf_rotate(const etf_ctx *ctx, const float *x, int64_t n, float *out)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->rotation.empty()) return fail(ctx, ETF_ESTATE, "no rotation: call etf_pq_set_rotation or etf_opq_train first");
    if (n < 0 || (n > 0 && (!x || !out))) return fail(ctx, ETF_EINVAL, "null input or output with n=%lld", (long long)n);
    const int d = ctx->rot_d;
    const float *R = ctx->rotation.data();
    parallel_slices(n, host_threads(), [&](int, int64_t lo, int64_t hi) { rotate_rows(R, d, x, lo, hi, out); });
    return ETF_OK;
}

// inverse of a d x d matrix in place (Gauss-Jordan with partial pivoting); false if it is singular to working precision
static bool invert(std::vector<double> &a, int d)
{
    std::vector<double> inv((size_t)d * d, 0.0);
    for (int i = 0; i < d; ++i) inv[(size_t)i * d + i] = 1.0;
    for (int c = 0; c < d; ++c) {
        int p = c;
        for (int r = c + 1; r < d; ++r)
            if (std::fabs(a[(size_t)r * d + c]) > std::fabs(a[(size_t)p * d + c])) p = r;
        if (std::fabs(a[(size_t)p * d + c]) < 1e-300) return false;
        if (p != c)
            for (int j = 0; j < d; ++j) {
                std::swap(a[(size_t)p * d + j], a[(size_t)c * d + j]);
                std::swap(inv[(size_t)p * d + j], inv[(size_t)c * d + j]);
            }
        const double piv = 1.0 / a[(size_t)c * d + c];
        for (int j = 0; j < d; ++j) {
            a[(size_t)c * d + j] *= piv;
            inv[(size_t)c * d + j] *= piv;
        }
        parallel_slices(d, host_threads(), [&](int, int64_t lo, int64_t hi) {
            for (int64_t r = lo; r < hi; ++r) {
                if (r == c) continue;
                const double f = a[(size_t)r * d + c];
                if (f == 0.0) continue;
                for (int j = 0; j < d; ++j) {
                    a[(size_t)r * d + j] -= f * a[(size_t)c * d + j];
                    inv[(size_t)r * d + j] -= f * inv[(size_t)c * d + j];
                }
            }
        });
    }
    a.swap(inv);
    return true;
}

// The orthogonal matrix nearest to c (its polar factor U V^T for c = U S V^T), by Newton's iteration
// X <- (X + X^-T) / 2 from X = c scaled to unit Frobenius norm; false if c is singular.
static bool polar_factor(std::vector<double> &c, int d)
{
    double fro = 0.0;
    for (double v : c) fro += v * v;
    fro = std::sqrt(fro);
    if (!(fro > 0.0)) return false;
    for (double &v : c) v *= std::sqrt((double)d) / fro;
    for (int it = 0; it < 100; ++it) {
        std::vector<double> inv(c);
        if (!invert(inv, d)) return false;
        double change = 0.0;
        for (int i = 0; i < d; ++i)
            for (int j = 0; j < d; ++j) {
                const double nv = 0.5 * (c[(size_t)i * d + j] + inv[(size_t)j * d + i]);
                change = std::max(change, std::fabs(nv - c[(size_t)i * d + j]));
                c[(size_t)i * d + j] = nv;
            }
        if (change < 1e-13) break;
    }
    return true;
}

// Optimized product quantisation, the non-parametric alternation: with the rotation fixed, train the product
// quantiser on the rotated training set; with the quantiser fixed, the orthogonal R that minimises
// sum ||R x - decode(encode(R x))||^2 is the polar factor of sum yhat x^T.  The rotation starts from the one that is set
// (the identity if none) and ends up set together with the codebooks of the last round.
extern "C" int etf_opq_train(etf_ctx *ctx, const float *x, int64_t n, int d, int M, int K, int iters, int rounds, uint64_t seed)
{
    if (!ctx) return ETF_EINVAL;
    if (!x || n <= 0) return fail(ctx, ETF_EINVAL, "training set is empty or null");
    if (iters < 0 || rounds < 0) return fail(ctx, ETF_EINVAL, "iters and rounds must be >= 0");
    int rc = check_pq_shape(ctx, d, M, K);
    if (rc) return rc;
    try {
        if (ctx->rotation.empty() || ctx->rot_d != d) {
            ctx->rotation.assign((size_t)d * d, 0.f);
            for (int i = 0; i < d; ++i) ctx->rotation[(size_t)i * d + i] = 1.f;
            ctx->rot_d = d;
        }
        std::vector<float> y((size_t)n * d);
        std::vector<uint8_t> codes((size_t)n * M);
        const int ds = d / M;
        for (int round = 0;; ++round) {
            if ((rc = etf_rotate(ctx, x, n, y.data()))) return rc;
            if ((rc = etf_pq_train(ctx, y.data(), n, d, M, K, iters, seed))) return rc;
            if (round == rounds) break;
            if ((rc = etf_pq_encode(ctx, y.data(), n, codes.data()))) return rc;
            // c = sum over the training set of yhat x^T, in double
            const int threads = host_threads();
            std::vector<std::vector<double>> part((size_t)threads, std::vector<double>((size_t)d * d, 0.0));
            const float *cb = ctx->codebooks.data();
            parallel_slices(n, threads, [&](int t, int64_t lo, int64_t hi) {
                std::vector<double> &c = part[t];
                std::vector<float> yh((size_t)d);
                for (int64_t i = lo; i < hi; ++i) {
                    for (int m = 0; m < M; ++m)
                        memcpy(yh.data() + (size_t)m * ds, cb + ((size_t)m * K + codes[(size_t)i * M + m]) * ds, sizeof(float) * ds);
                    const float *xi = x + (size_t)i * d;
                    for (int r = 0; r < d; ++r) {
                        const double yr = yh[r];
                        double *cr = c.data() + (size_t)r * d;
                        for (int j = 0; j < d; ++j) cr[j] += yr * (double)xi[j];
                    }
                }
            });
            std::vector<double> c((size_t)d * d, 0.0);
            for (const auto &p : part)
                for (size_t i = 0; i < c.size(); ++i) c[i] += p[i];
            if (!polar_factor(c, d)) break;  // degenerate training set: keep the rotation of this round
            for (size_t i = 0; i < c.size(); ++i) ctx->rotation[i] = (float)c[i];
        }
    } catch (const std::bad_alloc &) {
        return fail(ctx, ETF_ENOMEM, "out of host memory");
    }
    return ETF_OK;
}

extern "C" int etf_pq_encode(const etf_ctx *ctx, const float *x, int64_t n, uint8_t *codes_out)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks: call etf_pq_train or etf_pq_set_codebooks first");
    if (n < 0 || (n > 0 && (!x || !codes_out))) return fail(ctx, ETF_EINVAL, "null input or output with n=%lld", (long long)n);
    const int d = ctx->d, M = ctx->M, K = ctx->K, ds = ctx->ds;
    const float *cb = ctx->codebooks.data();
    parallel_slices(n, host_threads(), [&](int, int64_t lo, int64_t hi) {
        for (int64_t i = lo; i < hi; ++i)
            for (int m = 0; m < M; ++m)
                codes_out[(size_t)i * M + m] =
                    (uint8_t)nearest_codeword(x + (size_t)i * d + (size_t)m * ds, cb + (size_t)m * K * ds, K, ds, nullptr);
    });
    return ETF_OK;
}

// =============================================================================================
// index build
// =============================================================================================
extern "C" int etf_index_build(etf_ctx *ctx, const uint8_t *codes, int64_t N, const int32_t *ids, int T,
                               const int32_t *chunk_begin)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks: M and K are unknown");
    const int M = ctx->M, K = ctx->K;
    if (!codes || N <= 0) return fail(ctx, ETF_EINVAL, "codes is null or N <= 0");
    if (N >= ((int64_t)1 << 31)) return fail(ctx, ETF_EINVAL, "N must be below 2^31");
    if (T < 1 || T > M) return fail(ctx, ETF_EINVAL, "need 1 <= T <= M (T=%d, M=%d)", T, M);
    if (!ctx->next_term.empty() && (int64_t)ctx->next_term.size() != N)
        return fail(ctx, ETF_EINVAL, "the leaf terms were given for %lld vectors, the build has %lld", (long long)ctx->next_term.size(), (long long)N);
    std::vector<int32_t> cb(T + 1);
    if (chunk_begin) {
        for (int t = 0; t <= T; ++t) cb[t] = chunk_begin[t];
        if (cb[0] != 0 || cb[T] != M) return fail(ctx, ETF_EINVAL, "chunk_begin must run from 0 to M");
        for (int t = 0; t < T; ++t)
            if (cb[t + 1] <= cb[t]) return fail(ctx, ETF_EINVAL, "chunk_begin must be strictly increasing");
    } else {
        if (M % T != 0) return fail(ctx, ETF_EINVAL, "T=%d does not divide M=%d and no chunk_begin was given", T, M);
        for (int t = 0; t <= T; ++t) cb[t] = t * (M / T);
    }
    {
        std::atomic<int> bad(0);
        parallel_slices(N, host_threads(), [&](int, int64_t lo, int64_t hi) {
            for (int64_t i = lo * M; i < hi * M; ++i)
                if (codes[i] >= K) { bad = 1; break; }
            if (ids)
                for (int64_t i = lo; i < hi; ++i)
                    if (ids[i] < 0) { bad = 2; break; }
        });
        if (bad == 1) return fail(ctx, ETF_EINVAL, "a code byte is >= K=%d", K);
        if (bad == 2) return fail(ctx, ETF_EINVAL, "ids must be non-negative");
    }
    try {
        HostIndex ix;
        ix.M = M; ix.K = K; ix.T = T; ix.N = N;
        ix.chunk_begin = cb;
        ix.order.resize(M);
        for (int j = 0; j < M; ++j) ix.order[j] = ctx->next_order.empty() ? j : ctx->next_order[j];
        ix.codes.resize((size_t)N * M);
        parallel_slices(N, host_threads(), [&](int, int64_t lo, int64_t hi) {
            for (int64_t i = lo; i < hi; ++i)
                for (int j = 0; j < M; ++j) ix.codes[(size_t)i * M + j] = codes[(size_t)i * M + ix.order[j]];
        });
        codes = ix.codes.data();  // from here on: the encodings in index order
        ix.ids_in.resize(N);
        for (int64_t i = 0; i < N; ++i) ix.ids_in[i] = ids ? ids[i] : (int32_t)i;
        ix.has_term = !ctx->next_term.empty();
        if (ix.has_term) ix.pterm = ctx->next_term;

        // 1. lexicographic sort of (encoding, id)  -- "in place sort of the encoded dataset"
        std::vector<KeyRec> rec((size_t)N);
        parallel_slices(N, host_threads(), [&](int, int64_t lo, int64_t hi) {
            for (int64_t i = lo; i < hi; ++i) {
                pack_key(codes + (size_t)i * M, 0, M, rec[i].k);
                rec[i].pos = (uint32_t)i;
                rec[i].id = ix.ids_in[i];
                uint32_t tb = 0;
                if (ix.has_term) memcpy(&tb, &ix.pterm[i], 4);
                rec[i].tb = tb;
            }
        });
        const int idbytes = ids ? 4 : 0;  // positions are already ascending when ids are implicit
        const int tbytes = ix.has_term ? 4 : 0;  // order: encoding, then term, then id
        radix_sort_records(rec, idbytes + tbytes + M, [idbytes, tbytes, M](const KeyRec &r, int p) -> int {
            if (p < idbytes) return (int)(((uint32_t)r.id >> (8 * p)) & 255);
            if (p < idbytes + tbytes) return (int)((r.tb >> (8 * (p - idbytes))) & 255);
            return key_byte(r.k, M - 1 - (p - idbytes - tbytes));
        });

        // 2. distinct encodings and their id ranges
        ix.ids_sorted.resize(N);
        ix.enc_of_pos.resize(N);
        ix.ebegin.clear();
        std::vector<KeyRec> distinct;  // key + pos = distinct number
        for (int64_t i = 0; i < N; ++i) {
            if (i == 0 || rec[i].k[0] != rec[i - 1].k[0] || rec[i].k[1] != rec[i - 1].k[1] || rec[i].tb != rec[i - 1].tb) {
                ix.ebegin.push_back((uint32_t)i);
                KeyRec r = rec[i];
                r.pos = (uint32_t)distinct.size();
                distinct.push_back(r);
            }
            ix.ids_sorted[i] = rec[i].id;
            ix.enc_of_pos[rec[i].pos] = (uint32_t)(distinct.size() - 1);
        }
        ix.ebegin.push_back((uint32_t)N);
        ix.Nd = (int64_t)distinct.size();
        ix.max_dup = 0;
        for (int64_t e = 0; e < ix.Nd; ++e) ix.max_dup = std::max<int64_t>(ix.max_dup, ix.ebegin[e + 1] - ix.ebegin[e]);
        ix.ecodes.resize((size_t)ix.Nd * M);
        for (int64_t e = 0; e < ix.Nd; ++e)
            for (int m = 0; m < M; ++m) ix.ecodes[(size_t)e * M + m] = (uint8_t)key_byte(distinct[e].k, m);
        if (ix.has_term) {
            ix.eterm.resize((size_t)ix.Nd);
            for (int64_t e = 0; e < ix.Nd; ++e) memcpy(&ix.eterm[e], &distinct[e].tb, 4);
        }
        { std::vector<KeyRec>().swap(rec); }

        // 3. one tree per chunk group
        ix.tree.assign(T, HostTree());
        for (int t = 0; t < T; ++t) {
            HostTree &tr = ix.tree[t];
            tr.c0 = cb[t];
            tr.D = cb[t + 1] - cb[t];
            if (T == 1 && !ix.has_term) {  // (with a payload several entries may share a leaf: the general path below)
                build_tree(distinct, tr.D, tr);
                continue;
            }
            std::vector<KeyRec> sub((size_t)ix.Nd);
            for (int64_t e = 0; e < ix.Nd; ++e) {
                pack_key(ix.ecodes.data() + (size_t)e * M, tr.c0, tr.c0 + tr.D, sub[e].k);
                sub[e].pos = (uint32_t)e;
                sub[e].id = 0;
            }
            if (t > 0) {  // tree 0 covers a prefix of the full encoding: already in order
                const int D = tr.D;
                radix_sort_records(sub, D, [D](const KeyRec &r, int p) -> int { return key_byte(r.k, D - 1 - p); });
            }
            tr.leaf_of.resize(ix.Nd);
            std::vector<KeyRec> uniq;
            for (int64_t i = 0; i < ix.Nd; ++i) {
                if (i == 0 || sub[i].k[0] != sub[i - 1].k[0] || sub[i].k[1] != sub[i - 1].k[1]) uniq.push_back(sub[i]);
                tr.leaf_of[sub[i].pos] = (uint32_t)(uniq.size() - 1);
            }
            { std::vector<KeyRec>().swap(sub); }
            build_tree(uniq, tr.D, tr);
        }

        // tree 0's chunks of every distinct encoding, as padded records (fused tree-0 / reduction kernel)
        {
            const int D0 = ix.tree[0].D;
            ix.rstride0 = std::max(4, depth_class(D0));
            ix.rec0.assign((size_t)ix.Nd * ix.rstride0, 0);
            const int pad = depth_class(D0) - D0;
            for (int64_t e = 0; e < ix.Nd; ++e)
                memcpy(ix.rec0.data() + (size_t)e * ix.rstride0 + pad, ix.ecodes.data() + (size_t)e * M, (size_t)D0);
        }

        // 4. threshold samples: a seeded random subset of the vectors (as encodings, and as positions)
        {
            uint64_t s = 0x1509051860ull ^ (uint64_t)N;
            auto sample_size = [&](int64_t n) { return etf::sample_size(ctx->opt, n); };
            int64_t want = sample_size(ix.Nd);
            int64_t S = std::min<int64_t>(ix.Nd, want);
            // The sample is stored in random order: consecutive runs of it are the sample groups whose
            // minima bound the k-th distance, and a group must not be a cluster of similar encodings.
            auto shuffle = [&s](std::vector<uint32_t> &v) {
                for (size_t i = v.size(); i > 1; --i) std::swap(v[i - 1], v[splitmix64(s) % i]);
            };
            if (S == ix.Nd) {
                ix.sample_enc.resize(S);
                for (int64_t i = 0; i < S; ++i) ix.sample_enc[i] = (uint32_t)i;
            } else {
                std::vector<uint32_t> v((size_t)S);
                for (int64_t i = 0; i < S; ++i) v[i] = ix.enc_of_pos[splitmix64(s) % (uint64_t)N];
                std::sort(v.begin(), v.end());
                v.erase(std::unique(v.begin(), v.end()), v.end());
                ix.sample_enc.swap(v);
            }
            shuffle(ix.sample_enc);
            want = sample_size(N);
            S = std::min<int64_t>(N, want);
            if (S == N) {
                ix.sample_pos.resize(S);
                for (int64_t i = 0; i < S; ++i) ix.sample_pos[i] = (uint32_t)i;
            } else {
                std::vector<uint32_t> v((size_t)S);
                for (int64_t i = 0; i < S; ++i) v[i] = (uint32_t)(splitmix64(s) % (uint64_t)N);
                std::sort(v.begin(), v.end());
                v.erase(std::unique(v.begin(), v.end()), v.end());
                ix.sample_pos.swap(v);
            }
            shuffle(ix.sample_pos);
            // the sampled encodings side by side in sample order, so that a kernel reads them as a stream
            ix.sample_enc_codes.resize(ix.sample_enc.size() * (size_t)M);
            for (size_t i = 0; i < ix.sample_enc.size(); ++i)
                memcpy(ix.sample_enc_codes.data() + i * M, ix.ecodes.data() + (size_t)ix.sample_enc[i] * M, (size_t)M);
            ix.sample_pos_codes.resize(ix.sample_pos.size() * (size_t)M);
            for (size_t i = 0; i < ix.sample_pos.size(); ++i)
                memcpy(ix.sample_pos_codes.data() + i * M, ix.codes.data() + (size_t)ix.sample_pos[i] * M, (size_t)M);
        }
        ix.n_sample_enc = (int64_t)ix.sample_enc.size();
        ix.n_sample_pos = (int64_t)ix.sample_pos.size();
        ix.built = true;
        ctx->idx = std::move(ix);
        ctx->dev_base = nullptr;
        ctx->next_term.clear();  // a payload belongs to one build
        compute_layout(ctx);
    } catch (const std::bad_alloc &) {
        drop_index(ctx);
        return fail(ctx, ETF_ENOMEM, "out of host memory while building the index");
    }
    return ETF_OK;
}

// =============================================================================================
// leaf payload
// =============================================================================================
extern "C" int etf_index_set_leaf_term(etf_ctx *ctx, const float *term, int64_t N)
{
    if (!ctx) return ETF_EINVAL;
    if (!term) {
        ctx->next_term.clear();
        return ETF_OK;
    }
    if (N <= 0) return fail(ctx, ETF_EINVAL, "N must be positive");
    for (int64_t i = 0; i < N; ++i)
        if (!(term[i] >= 0.f) || !(term[i] <= 3.0e38f)) return fail(ctx, ETF_EINVAL, "leaf term %lld is negative or not finite", (long long)i);
    try {
        ctx->next_term.resize((size_t)N);
        for (int64_t i = 0; i < N; ++i) ctx->next_term[i] = term[i] == 0.f ? 0.f : term[i];  // -0 becomes +0: one bit pattern per value
    } catch (const std::bad_alloc &) {
        ctx->next_term.clear();
        return fail(ctx, ETF_ENOMEM, "out of host memory");
    }
    return ETF_OK;
}

extern "C" int etf_index_set_leaf_bytes(etf_ctx *ctx, const uint8_t *bytes, int64_t N, float scale, float offset)
{
    if (!ctx) return ETF_EINVAL;
    if (!bytes) return etf_index_set_leaf_term(ctx, nullptr, 0);
    if (N <= 0) return fail(ctx, ETF_EINVAL, "N must be positive");
    try {
        std::vector<float> t((size_t)N);
        for (int64_t i = 0; i < N; ++i) t[i] = fmaf(scale, (float)bytes[i], offset);
        return etf_index_set_leaf_term(ctx, t.data(), N);
    } catch (const std::bad_alloc &) {
        return fail(ctx, ETF_ENOMEM, "out of host memory");
    }
}

// =============================================================================================
// chunk order
// =============================================================================================
static int check_order(const etf_ctx *ctx, const int32_t *order)
{
    const int M = ctx->M;
    bool seen[ETF_MAX_M] = {false};
    for (int j = 0; j < M; ++j) {
        if (order[j] < 0 || order[j] >= M || seen[order[j]]) return fail(ctx, ETF_EINVAL, "order must be a permutation of 0..%d", M - 1);
        seen[order[j]] = true;
    }
    return ETF_OK;
}

extern "C" int etf_index_set_chunk_order(etf_ctx *ctx, const int32_t *order)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks: M is unknown");
    if (!order) {
        ctx->next_order.clear();
        return ETF_OK;
    }
    int rc = check_order(ctx, order);
    if (rc) return rc;
    ctx->next_order.assign(order, order + ctx->M);
    return ETF_OK;
}

// table lookups of one traversal of the index of `codes` in the given order
static int count_lookups(const etf_ctx *ctx, const uint8_t *codes, int64_t n, int T, const int32_t *chunk_begin,
                         const int32_t *order, int64_t *out)
{
    etf_ctx tmp;
    tmp.d = ctx->d; tmp.M = ctx->M; tmp.K = ctx->K; tmp.ds = ctx->ds;
    tmp.codebooks.assign(1, 0.f);  // the builder only asks whether a quantiser is set
    tmp.opt = ctx->opt;
    if (order) tmp.next_order.assign(order, order + ctx->M);
    int rc = etf_index_build(&tmp, codes, n, nullptr, T, chunk_begin);
    if (rc) return fail(ctx, rc, "%s", tmp.err.c_str());
    etf_stats st;
    rc = etf_index_stats(&tmp, &st);
    if (rc) return fail(ctx, rc, "%s", tmp.err.c_str());
    *out = 0;
    for (int t = 0; t < T; ++t) *out += st.lookups[t];
    return ETF_OK;
}

extern "C" int etf_suggest_chunk_order(const etf_ctx *ctx, const uint8_t *codes, int64_t N, int T, const int32_t *chunk_begin,
                                       int32_t *order_out, int64_t *lookups_given, int64_t *lookups_order)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks: M and K are unknown");
    const int M = ctx->M;
    if (!codes || N <= 0 || !order_out) return fail(ctx, ETF_EINVAL, "codes or order_out is null, or N <= 0");
    if (T < 1 || T > M) return fail(ctx, ETF_EINVAL, "need 1 <= T <= M (T=%d, M=%d)", T, M);
    std::vector<int32_t> cb(T + 1);
    if (chunk_begin) {
        for (int t = 0; t <= T; ++t) cb[t] = chunk_begin[t];
        if (cb[0] != 0 || cb[T] != M) return fail(ctx, ETF_EINVAL, "chunk_begin must run from 0 to M");
        for (int t = 0; t < T; ++t)
            if (cb[t + 1] <= cb[t]) return fail(ctx, ETF_EINVAL, "chunk_begin must be strictly increasing");
    } else {
        if (M % T != 0) return fail(ctx, ETF_EINVAL, "T=%d does not divide M=%d and no chunk_begin was given", T, M);
        for (int t = 0; t <= T; ++t) cb[t] = t * (M / T);
    }
    try {
        // evenly spaced sample
        const int64_t cap = (int64_t)1 << 18;
        const int64_t step = (N + cap - 1) / cap, n = (N + step - 1) / step;
        std::vector<uint8_t> rows((size_t)n * M);
        for (int64_t i = 0; i < n; ++i) memcpy(rows.data() + (size_t)i * M, codes + (size_t)(i * step) * M, (size_t)M);
        for (size_t i = 0; i < rows.size(); ++i)
            if (rows[i] >= ctx->K) return fail(ctx, ETF_EINVAL, "a code byte is >= K=%d", ctx->K);
        std::vector<bool> used(M, false);
        std::vector<uint32_t> gid((size_t)n);
        int pos = 0;
        for (int t = 0; t < T; ++t) {
            std::fill(gid.begin(), gid.end(), 0u);  // every tree starts from the empty prefix
            for (int l = cb[t]; l < cb[t + 1]; ++l, ++pos) {
                // distinct (prefix so far, chunk c) pairs for every remaining chunk c
                std::vector<int64_t> distinct(M, -1);
                std::vector<int> cand;
                for (int c = 0; c < M; ++c)
                    if (!used[c]) cand.push_back(c);
                parallel_slices((int64_t)cand.size(), host_threads(), [&](int, int64_t lo, int64_t hi) {
                    std::vector<uint64_t> keys((size_t)n);
                    for (int64_t ci = lo; ci < hi; ++ci) {
                        const int c = cand[ci];
                        for (int64_t i = 0; i < n; ++i) keys[i] = ((uint64_t)gid[i] << 8) | rows[(size_t)i * M + c];
                        std::sort(keys.begin(), keys.end());
                        distinct[c] = (int64_t)(std::unique(keys.begin(), keys.end()) - keys.begin());
                    }
                });
                int best = cand[0];
                for (int c : cand)
                    if (distinct[c] < distinct[best]) best = c;  // ties: the lowest chunk number
                used[best] = true;
                order_out[pos] = best;
                // the prefixes one level further down, numbered densely
                std::vector<uint64_t> keys((size_t)n);
                for (int64_t i = 0; i < n; ++i) keys[i] = ((uint64_t)gid[i] << 8) | rows[(size_t)i * M + best];
                std::vector<uint64_t> uniq(keys);
                std::sort(uniq.begin(), uniq.end());
                uniq.erase(std::unique(uniq.begin(), uniq.end()), uniq.end());
                for (int64_t i = 0; i < n; ++i) gid[i] = (uint32_t)(std::lower_bound(uniq.begin(), uniq.end(), keys[i]) - uniq.begin());
            }
        }
        // the greedy choice looks one level ahead only: keep the given order unless the suggestion saves lookups
        int64_t given = 0, suggested = 0;
        int rc;
        if ((rc = count_lookups(ctx, rows.data(), n, T, cb.data(), nullptr, &given))) return rc;
        if ((rc = count_lookups(ctx, rows.data(), n, T, cb.data(), order_out, &suggested))) return rc;
        if (suggested >= given) {
            for (int j = 0; j < M; ++j) order_out[j] = j;
            suggested = given;
        }
        if (lookups_given) *lookups_given = given;
        if (lookups_order) *lookups_order = suggested;
    } catch (const std::bad_alloc &) {
        return fail(ctx, ETF_ENOMEM, "out of host memory while choosing the chunk order");
    }
    return ETF_OK;
}

// Which chunks form a tree (paper, "Encoding Forests" and its remark on future work): for T trees, the cut of the M
// positions into T contiguous groups, together with the greedy chunk order for that cut, whose index needs the fewest
// table lookups per traversal.  All cuts are tried while there are at most 64 of them; otherwise a descent from the
// equal cut that moves one boundary by one position as long as that saves lookups.
extern "C" int etf_suggest_partition(const etf_ctx *ctx, const uint8_t *codes, int64_t N, int T, int32_t *chunk_begin_out,
                                     int32_t *order_out, int64_t *lookups_equal, int64_t *lookups_best)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks: M and K are unknown");
    const int M = ctx->M;
    if (!codes || N <= 0 || !order_out || !chunk_begin_out) return fail(ctx, ETF_EINVAL, "codes, chunk_begin_out or order_out is null, or N <= 0");
    if (T < 1 || T > M) return fail(ctx, ETF_EINVAL, "need 1 <= T <= M (T=%d, M=%d)", T, M);
    try {
        // the trial indexes are built on at most 2^16 evenly spaced vectors (etf_suggest_chunk_order samples its input again)
        const int64_t cap = (int64_t)1 << 16;
        const int64_t step = (N + cap - 1) / cap, n = (N + step - 1) / step;
        std::vector<uint8_t> rows((size_t)n * M);
        for (int64_t i = 0; i < n; ++i) memcpy(rows.data() + (size_t)i * M, codes + (size_t)(i * step) * M, (size_t)M);
        std::vector<int32_t> order(M);
        auto cost_of = [&](const std::vector<int32_t> &cb, std::vector<int32_t> &ord, int64_t &cost) -> int {
            int64_t given = 0;
            return etf_suggest_chunk_order(ctx, rows.data(), n, T, cb.data(), ord.data(), &given, &cost);
        };
        // the (nearly) equal cut: the reference
        std::vector<int32_t> best_cb(T + 1), best_order(M);
        for (int t = 0; t <= T; ++t) best_cb[t] = (int32_t)((int64_t)t * M / T);
        int64_t best = 0;
        int rc = cost_of(best_cb, best_order, best);
        if (rc) return rc;
        const int64_t equal = best;
        // number of cuts: C(M - 1, T - 1)
        double ncuts = 1.0;
        for (int i = 1; i <= T - 1; ++i) ncuts = ncuts * (M - T + i) / i;
        if (ncuts <= 64.0) {
            std::vector<int32_t> cb(T + 1);
            cb[0] = 0;
            cb[T] = M;
            // boundaries 1 <= b_1 < ... < b_{T-1} <= M - 1, in lexicographic order
            std::vector<int32_t> b(T - 1);
            for (int i = 0; i < T - 1; ++i) b[i] = i + 1;
            for (;;) {
                for (int i = 0; i < T - 1; ++i) cb[i + 1] = b[i];
                int64_t c = 0;
                if ((rc = cost_of(cb, order, c))) return rc;
                if (c < best) {
                    best = c;
                    best_cb = cb;
                    best_order = order;
                }
                int i = T - 2;
                while (i >= 0 && b[i] == M - (T - 1) + i) --i;
                if (i < 0) break;
                ++b[i];
                for (int j = i + 1; j < T - 1; ++j) b[j] = b[j - 1] + 1;
            }
        } else {
            bool moved = true;
            while (moved) {
                moved = false;
                for (int i = 1; i < T; ++i)
                    for (int dlt = -1; dlt <= 1; dlt += 2) {
                        std::vector<int32_t> cb = best_cb;
                        cb[i] += dlt;
                        if (cb[i] <= cb[i - 1] || cb[i] >= cb[i + 1]) continue;
                        int64_t c = 0;
                        if ((rc = cost_of(cb, order, c))) return rc;
                        if (c < best) {
                            best = c;
                            best_cb = cb;
                            best_order = order;
                            moved = true;
                        }
                    }
            }
        }
        for (int t = 0; t <= T; ++t) chunk_begin_out[t] = best_cb[t];
        for (int j = 0; j < M; ++j) order_out[j] = best_order[j];
        if (lookups_equal) *lookups_equal = equal;
        if (lookups_best) *lookups_best = best;
    } catch (const std::bad_alloc &) {
        return fail(ctx, ETF_ENOMEM, "out of host memory while choosing the partition");
    }
    return ETF_OK;
}

extern "C" int etf_index_stats(const etf_ctx *ctx, etf_stats *out)
{
    if (!ctx) return ETF_EINVAL;
    if (!out) return fail(ctx, ETF_EINVAL, "output pointer is null");
    if (!ctx->idx.built) return fail(ctx, ETF_ESTATE, "no index: call etf_index_build first");
    const HostIndex &ix = ctx->idx;
    memset(out, 0, sizeof *out);
    out->M = ix.M; out->K = ix.K; out->T = ix.T;
    for (int t = 0; t <= ix.T; ++t) out->chunk_begin[t] = ix.chunk_begin[t];
    out->N = ix.N; out->n_distinct = ix.Nd; out->max_dup = ix.max_dup;
    for (int t = 0; t < ix.T; ++t) {
        const HostTree &tr = ix.tree[t];
        for (int l = 0; l < tr.D; ++l) {
            out->nI[t][l] = tr.nI[l];
            out->nL[t][l] = tr.nL[l];
            out->L1[t] += out->nI[t][l];
            out->L2[t] += out->nL[t][l];
            out->sumP[t] += out->nL[t][l] * (tr.D - (l + 1));
        }
        out->lookups[t] = out->L1[t] + out->L2[t] + out->sumP[t];
        out->paper_bytes[t] = 4 * ix.N + 2 * (out->L1[t] + out->L2[t]) + out->sumP[t];
    }
    out->device_bytes = ctx->lay.total;
    for (int j = 0; j < ix.M; ++j) out->chunk_order[j] = ix.order[j];
    return ETF_OK;
}

extern "C" int64_t etf_index_device_bytes(const etf_ctx *ctx)
{
    if (!ctx) return ETF_EINVAL;
    if (!ctx->idx.built) return fail(ctx, ETF_ESTATE, "no index: call etf_index_build first");
    return ctx->lay.total;
}

extern "C" int etf_index_layout(const etf_ctx *ctx, etf_layout *out)
{
    if (!ctx) return ETF_EINVAL;
    if (!out) return fail(ctx, ETF_EINVAL, "output pointer is null");
    if (!ctx->idx.built) return fail(ctx, ETF_ESTATE, "no index: call etf_index_build first");
    const HostIndex &ix = ctx->idx;
    const DevLayout &L = ctx->lay;
    memset(out, 0xFF, sizeof *out);  // every offset -1 unless set below
    out->total = L.total;
    out->codebooks = L.codebooks; out->codes = L.codes; out->ids_in = L.ids_in; out->ids_sorted = L.ids_sorted;
    out->ebegin = L.ebegin; out->enc_of_pos = L.enc_of_pos; out->ecodes = L.ecodes;
    out->sample_enc = L.sample_enc; out->sample_pos = L.sample_pos;
    out->sample_enc_codes = L.sample_enc_codes; out->sample_pos_codes = L.sample_pos_codes;
    out->rec0 = L.rec0;
    out->cb_centered = L.cb_centered; out->cb_norm = L.cb_norm; out->cb_mean = L.cb_mean;
    out->cb_row = ctx->dsp;
    out->eterm = L.eterm;
    out->pterm = L.pterm;
    out->rec0_stride = ix.rstride0;
    out->n_sample_enc = ix.n_sample_enc;
    out->n_sample_pos = ix.n_sample_pos;
    for (int t = 0; t < ix.T; ++t) {
        out->leaf_of[t] = L.tree[t].leaf_of;
        out->trec[t] = L.tree[t].rec;
        out->trec_stride[t] = ix.tree[t].rstride;
        for (int l = 0; l < ix.tree[t].D; ++l) {
            out->icode[t][l] = L.tree[t].icode[l];
            out->iparent[t][l] = L.tree[t].iparent[l];
            out->lcodes[t][l] = L.tree[t].lcodes[l];
            out->lparent[t][l] = L.tree[t].lparent[l];
            out->lrow[t][l] = L.tree[t].lrow[l];
            out->lstride[t][l] = ix.tree[t].bucket[l].stride;
        }
    }
    return ETF_OK;
}

extern "C" int etf_index_export(const etf_ctx *ctx, void *host_buf, int64_t bytes)
{
    if (!ctx) return ETF_EINVAL;
    if (!host_buf) return fail(ctx, ETF_EINVAL, "output pointer is null");
    if (!ctx->idx.built) return fail(ctx, ETF_ESTATE, "no index: call etf_index_build first");
    if (ctx->idx.device_built) return fail(ctx, ETF_ESTATE, "the index was built on the device: the host holds no copy of it");
    if (bytes < ctx->lay.total) return fail(ctx, ETF_ENOMEM, "buffer too small: %lld < %lld", (long long)bytes, (long long)ctx->lay.total);
    memset(host_buf, 0, (size_t)ctx->lay.total);
    char *base = (char *)host_buf;
    for_each_image_array(ctx, [base](int64_t off, const void *src, size_t n) {
        if (n) memcpy(base + off, src, n);
    });
    return ETF_OK;
}
