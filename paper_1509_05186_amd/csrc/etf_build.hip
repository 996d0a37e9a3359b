// Index build on the device (Algorithm 1; the remark on building in parallel that closes "Efficient Encoding Tree
// Construction"): the lexicographic sort of the encodings, the merge of repeated encodings into id ranges, every
// tree's level arrays from the longest common prefixes of neighbouring sorted (sub-)encodings, and the threshold
// samples.  The sorts and the prefix sums are rocPRIM's device-wide radix sort and scan; everything around them is
// kernels of this file.  The image has the layout the host builder's has (the same layout function, fed with the
// counts as they come back from the device), so the two are interchangeable byte for byte, samples aside.
#include <cstring>

#include <hip/hip_runtime.h>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>

#include <algorithm>
#include <numeric>

#include "etf_internal.h"

using namespace etf;

#define HIP_TRY(ctx, call)                                                                            \
    do {                                                                                              \
        hipError_t e_ = (call);                                                                       \
        if (e_ != hipSuccess) return fail(ctx, ETF_EHIP, "%s: %s", #call, hipGetErrorString(e_));     \
    } while (0)

namespace {

constexpr int BT = 256;  // threads per workgroup of every kernel here

inline int64_t al256(int64_t x) { return (x + 255) & ~(int64_t)255; }
inline unsigned blocks(int64_t n) { return (unsigned)((n + BT - 1) / BT); }

// scal[0] = distinct encodings, scal[1] = largest number of vectors sharing one encoding, scal[2] = input faults
// (bit 0: a code byte >= K, bit 1: a negative id)
__global__ void __launch_bounds__(BT) k_build_init(const uint8_t *codes, const int32_t *ids, int64_t N, int M, int K,
                                                   uint32_t *pos, int32_t *ids_in, uint32_t *scal)
{
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i == 0) {
        scal[0] = 0;
        scal[1] = 0;
    }
    if (i >= N) return;
    pos[i] = (uint32_t)i;
    const int32_t id = ids ? ids[i] : (int32_t)i;
    ids_in[i] = id;
    uint32_t bad = id < 0 ? 2u : 0u;
    if (K < 256)
        for (int m = 0; m < M; ++m)
            if (codes[i * M + m] >= K) bad |= 1u;
    if (bad) atomicOr(&scal[2], bad);
}

// the input encodings in index order: position j holds input chunk src[j] (a thread reads its whole row before it
// writes: in and out may be the same buffer)
struct BuildOrder {
    uint8_t src[ETF_MAX_M];
};

__global__ void __launch_bounds__(BT) k_build_permute(const uint8_t *in, uint8_t *out, int64_t N, int M, BuildOrder ord)
{
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i >= N) return;
    uint8_t row[ETF_MAX_M];
#pragma unroll
    for (int j = 0; j < ETF_MAX_M; ++j) row[j] = j < M ? in[i * M + j] : (uint8_t)0;
    uint8_t res[ETF_MAX_M];
#pragma unroll
    for (int j = 0; j < ETF_MAX_M; ++j) {
        uint8_t v = 0;
#pragma unroll
        for (int c = 0; c < ETF_MAX_M; ++c) v = ord.src[j] == c ? row[c] : v;
        res[j] = v;
    }
#pragma unroll
    for (int j = 0; j < ETF_MAX_M; ++j)
        if (j < M) out[i * M + j] = res[j];
}

// Sort key of row pos[i]: chunks [c0, c1) of it (at most eight), most significant first, so that integer order is
// lexicographic order, in the low 8 (c1 - c0) bits (the sort then leaves out the empty high bits); c0 == c1 asks
// for the row's id instead.
__global__ void __launch_bounds__(BT) k_build_keys(const uint8_t *rows, int M, const int32_t *ids_in, const uint32_t *pos,
                                                   int64_t N, int c0, int c1, uint64_t *keys)
{
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i >= N) return;
    const int64_t p = pos[i];
    uint64_t k = 0;
    if (c0 == c1) {
        k = (uint64_t)(uint32_t)ids_in[p];
    } else {
        for (int c = c0; c < c1; ++c) k |= (uint64_t)rows[p * M + c] << (8 * (c1 - 1 - c));
    }
    keys[i] = k;
}

__global__ void __launch_bounds__(BT) k_build_iota(uint32_t *pos, int64_t N)
{
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i < N) pos[i] = (uint32_t)i;
}

// head[i] = 1 where the i-th row in sorted order differs from its predecessor in chunks [c0, c0 + D)
__global__ void __launch_bounds__(BT) k_build_heads(const uint8_t *rows, const uint32_t *pos, int64_t N, int M, int c0, int D,
                                                    uint32_t *head)
{
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i >= N) return;
    uint32_t h = 1;
    if (i > 0) {
        const uint8_t *a = rows + (int64_t)pos[i] * M + c0, *b = rows + (int64_t)pos[i - 1] * M + c0;
        h = 0;
        for (int m = 0; m < D; ++m) h |= a[m] != b[m];
    }
    head[i] = h;
}

// rank[i] = inclusive prefix sum of head: the i-th sorted vector has distinct-encoding number rank[i] - 1
__global__ void __launch_bounds__(BT) k_build_scatter(const uint8_t *codes, const int32_t *ids_in, const uint32_t *pos,
                                                      const uint32_t *head, const uint32_t *rank, int64_t N, int M,
                                                      int32_t *ids_sorted, uint32_t *enc_of_pos, uint32_t *ebegin,
                                                      uint8_t *ecodes, uint32_t *scal)
{
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i >= N) return;
    const int64_t p = pos[i];
    const uint32_t e = rank[i] - 1;
    ids_sorted[i] = ids_in[p];
    enc_of_pos[p] = e;
    if (head[i]) {
        ebegin[e] = (uint32_t)i;
        for (int m = 0; m < M; ++m) ecodes[(int64_t)e * M + m] = codes[p * M + m];
    }
    if (i == N - 1) {
        ebegin[e + 1] = (uint32_t)N;
        scal[0] = e + 1;
    }
}

__global__ void __launch_bounds__(BT) k_build_maxdup(const uint32_t *ebegin, uint32_t *scal)
{
    const int64_t e = (int64_t)blockIdx.x * BT + threadIdx.x;
    uint32_t n = e < (int64_t)scal[0] ? ebegin[e + 1] - ebegin[e] : 0;
    for (int o = 32; o > 0; o >>= 1) n = max(n, (uint32_t)__shfl_xor((int)n, o));
    // one atomic per wave, and only where it can still raise the maximum (the plain read may be stale: it only
    // filters; almost every wave then skips the contended address)
    if ((threadIdx.x & 63) == 0 && n > *(volatile uint32_t *)&scal[1]) atomicMax(&scal[1], n);
}

// ---- one tree over chunks [c0, c0 + D) of the distinct encodings -------------------------------------------------
// eord: the distinct encodings in the order of their sub-encoding; head/rank as above over that order.  Writes the
// leaf number of every distinct encoding and the distinct sub-encodings as records padded at the front.
__global__ void __launch_bounds__(BT) k_tree_records(const uint8_t *ecodes, int M, int c0, int D, const uint32_t *eord,
                                                     const uint32_t *head, const uint32_t *rank, int64_t Nd,
                                                     uint32_t *leaf_of, uint8_t *rec, int rstride, int pad)
{
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i >= Nd) return;
    const int64_t e = eord[i];
    const uint32_t u = rank[i] - 1;
    if (leaf_of) leaf_of[e] = u;
    if (head[i]) {
        uint8_t *r = rec + (int64_t)u * rstride;
        for (int j = 0; j < rstride; ++j) r[j] = (j >= pad && j < pad + D) ? ecodes[e * M + c0 + j - pad] : (uint8_t)0;
    }
}

// lcp[u] = chunks the u-th sorted sub-encoding shares with its predecessor; lcp[0] = lcp[U] = 0
__global__ void __launch_bounds__(BT) k_tree_lcp(const uint8_t *rec, int rstride, int pad, int D, int64_t U, uint8_t *lcp)
{
    const int64_t u = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (u > U) return;
    int n = 0;
    if (u > 0 && u < U) {
        const uint8_t *a = rec + u * rstride + pad, *b = a - rstride;
        while (n < D && a[n] == b[n]) ++n;
    }
    lcp[u] = (uint8_t)n;
}

// Level l (1-based): a prefix group of length l starts at u where lcp[u] < l; it is an internal node when the next
// sub-encoding still shares it (lcp[u + 1] >= l; only below the last level); u is a leaf of the level at which
// it is alone in its group, 1 + max(lcp[u], lcp[u + 1]).  flags = internal | leaf << 32: one scan numbers both.
__global__ void __launch_bounds__(BT) k_tree_flags(const uint8_t *lcp, int64_t U, int l, int D, uint64_t *flags)
{
    const int64_t u = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (u >= U) return;
    const int a = lcp[u], b = lcp[u + 1];
    const uint64_t internal = (l < D && a < l && b >= l) ? 1u : 0u;
    const uint64_t leaf = (1 + max(a, b) == l) ? 1u : 0u;
    flags[u] = internal | (leaf << 32);
}

// cur / prev: inclusive scans of this level's and the previous level's flags.  The parent of a node that starts
// at u is the last internal node of the previous level that starts at or before u (u's own group there: it holds
// at least two sub-encodings, or u would be a leaf higher up).
__global__ void __launch_bounds__(BT) k_tree_level(const uint8_t *rec, int rstride, int pad, int D, const uint8_t *lcp,
                                                   const uint64_t *cur, const uint64_t *prev, int64_t U, int l,
                                                   uint8_t *icode, uint32_t *iparent, uint8_t *lcodes, int lstride,
                                                   uint32_t *lparent, uint32_t *lrow)
{
    const int64_t u = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (u >= U) return;
    const int a = lcp[u], b = lcp[u + 1];
    const uint32_t parent = l > 1 ? (uint32_t)(prev[u] & 0xFFFFFFFFu) - 1u : 0xFFFFFFFFu;
    const uint8_t *r = rec + u * rstride + pad;
    if (l < D && a < l && b >= l) {
        const uint32_t n = (uint32_t)(cur[u] & 0xFFFFFFFFu) - 1u;
        icode[n] = r[l - 1];
        iparent[n] = parent;
    }
    if (1 + max(a, b) == l) {
        const uint32_t n = (uint32_t)(cur[u] >> 32) - 1u;
        for (int j = 0; j < lstride; ++j) lcodes[(int64_t)n * lstride + j] = j < D - l + 1 ? r[l - 1 + j] : (uint8_t)0;
        lparent[n] = parent;
        lrow[n] = (uint32_t)u;
    }
}

// tree 0's chunks of every distinct encoding as records padded at the front
__global__ void __launch_bounds__(BT) k_build_rec0(const uint8_t *ecodes, int M, int D0, int64_t Nd, uint8_t *rec0, int rstride, int pad)
{
    const int64_t e = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (e >= Nd) return;
    for (int j = 0; j < rstride; ++j) rec0[e * rstride + j] = (j >= pad && j < pad + D0) ? ecodes[e * M + j - pad] : (uint8_t)0;
}

__device__ inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// A sample of S of n rows without repeats: [0, n) is cut into S strata of (almost) equal length and one row is
// drawn from each.  Slot i of the sample holds stratum (i * A + B) mod S, A coprime to S: neighbouring slots (and
// with them the sample groups the kernels cut the sample into) hold rows from all over the range.
__global__ void __launch_bounds__(BT) k_build_sample(const uint8_t *rows, int64_t n, int M, int64_t S, uint64_t A, uint64_t B,
                                                     uint64_t seed, uint32_t *out_idx, uint8_t *out_rows)
{
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i >= S) return;
    const uint64_t s = ((uint64_t)i * A + B) % (uint64_t)S;  // S < 2^31, A < S: no overflow
    const uint64_t lo = s * (uint64_t)n / (uint64_t)S, hi = (s + 1) * (uint64_t)n / (uint64_t)S;  // n < 2^31 too
    const uint64_t r = lo + mix64(seed ^ s) % (hi - lo);  // S <= n: every stratum holds a row
    out_idx[i] = (uint32_t)r;
    for (int m = 0; m < M; ++m) out_rows[i * M + m] = rows[r * M + m];
}

// The sample of distinct encodings behind the bound of the tree modes, drawn through the vectors: the N vectors in
// sorted order are cut into S0 strata, one vector is drawn from each, and the draw stands for its encoding, found by
// bisection in ebegin.  An encoding is then drawn in proportion to the number of vectors that have it, which for
// queries that fall where the database is dense gives a much tighter bound than drawing every encoding equally
// (the bound counts vectors).  Draws of one encoding come from neighbouring strata; keep[s] = 1 marks the first.
__device__ inline uint32_t stratum_encoding(const uint32_t *ebegin, int64_t Nd, int64_t N, int64_t S0, uint64_t seed, uint64_t s)
{
    const uint64_t lo = s * (uint64_t)N / (uint64_t)S0, hi = (s + 1) * (uint64_t)N / (uint64_t)S0;
    const uint32_t r = (uint32_t)(lo + mix64(seed ^ s) % (hi - lo));  // S0 <= N: every stratum holds a vector
    int64_t a = 0, b = Nd;  // the e with ebegin[e] <= r < ebegin[e + 1]
    while (b - a > 1) {
        const int64_t mid = (a + b) >> 1;
        if (ebegin[mid] <= r) a = mid; else b = mid;
    }
    return (uint32_t)a;
}

__global__ void __launch_bounds__(BT) k_build_sample_draw(const uint32_t *ebegin, int64_t Nd, int64_t N, int64_t S0, uint64_t seed,
                                                          uint32_t *draw, uint32_t *keep)
{
    const int64_t s = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (s >= S0) return;
    const uint32_t e = stratum_encoding(ebegin, Nd, N, S0, seed, (uint64_t)s);
    draw[s] = e;
    keep[s] = (s == 0 || stratum_encoding(ebegin, Nd, N, S0, seed, (uint64_t)s - 1) != e) ? 1u : 0u;
}

// The kept draws in scattered order: the j-th kept draw (kscan[s] - 1, in sorted order) goes to slot i with
// j = (i * A + B) mod S, i.e. i = (j - B) * Ainv mod S, so that neighbouring slots hold encodings from all over the range.
__global__ void __launch_bounds__(BT) k_build_sample_place(const uint32_t *draw, const uint32_t *keep, const uint32_t *kscan, int64_t S0,
                                                           int64_t S, uint64_t Ainv, uint64_t B, const uint8_t *ecodes, int M,
                                                           uint32_t *out_idx, uint8_t *out_rows)
{
    const int64_t s = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (s >= S0 || !keep[s]) return;
    const uint64_t j = kscan[s] - 1u;
    const uint64_t i = ((j + (uint64_t)S - B % (uint64_t)S) % (uint64_t)S) * Ainv % (uint64_t)S;  // S < 2^31: no overflow
    const uint32_t e = draw[s];
    out_idx[i] = e;
    for (int m = 0; m < M; ++m) out_rows[i * M + m] = ecodes[(int64_t)e * M + m];
}

// multiplier of the slot -> stratum map: near S / golden ratio, coprime to S
// a^-1 mod S for a coprime to S (extended Euclid), 0 for S = 1
uint64_t inverse_mod(uint64_t a, int64_t S)
{
    if (S <= 1) return 0;
    int64_t t = 0, nt = 1, r = S, nr = (int64_t)(a % (uint64_t)S);
    while (nr != 0) {
        const int64_t q = r / nr;
        const int64_t t2 = t - q * nt, r2 = r - q * nr;
        t = nt; nt = t2; r = nr; nr = r2;
    }
    return (uint64_t)(t < 0 ? t + S : t);
}

uint64_t spread_multiplier(int64_t S)
{
    if (S <= 2) return 1;
    int64_t a = (int64_t)((double)S * 0.6180339887498949);
    a = std::max<int64_t>(1, std::min(a, S - 1));
    while (std::gcd(a, S) != 1) ++a;  // S - 1 is coprime to S: the loop ends below S
    return (uint64_t)a;
}

struct BuildWs {
    int64_t keys[2], pos[2], head, rank, scal, lcp, flags, scan[2], temp, temp_bytes, total;
};

int plan_ws(const etf_ctx *ctx, int64_t N, BuildWs &W)
{
    size_t t_sort = 0, t_scan = 0, t_scan64 = 0;
    // size queries: no launch, no device memory touched
    hipError_t e = rocprim::radix_sort_pairs(nullptr, t_sort, (uint64_t *)nullptr, (uint64_t *)nullptr, (uint32_t *)nullptr,
                                             (uint32_t *)nullptr, (size_t)N, 0u, 64u, (hipStream_t)ctx->stream);
    if (e != hipSuccess) return fail(ctx, ETF_EHIP, "radix sort size query: %s", hipGetErrorString(e));
    e = rocprim::inclusive_scan(nullptr, t_scan, (uint32_t *)nullptr, (uint32_t *)nullptr, (size_t)N, rocprim::plus<uint32_t>(),
                                (hipStream_t)ctx->stream);
    if (e != hipSuccess) return fail(ctx, ETF_EHIP, "scan size query: %s", hipGetErrorString(e));
    e = rocprim::inclusive_scan(nullptr, t_scan64, (uint64_t *)nullptr, (uint64_t *)nullptr, (size_t)N, rocprim::plus<uint64_t>(),
                                (hipStream_t)ctx->stream);
    if (e != hipSuccess) return fail(ctx, ETF_EHIP, "scan size query: %s", hipGetErrorString(e));
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        int64_t o = off;
        off = al256(off + std::max<int64_t>(bytes, 4));
        return o;
    };
    W.keys[0] = take(N * 8);
    W.keys[1] = take(N * 8);
    W.pos[0] = take(N * 4);
    W.pos[1] = take(N * 4);
    W.head = take(N * 4);
    W.rank = take(N * 4);
    W.scal = take(16);
    W.lcp = take(N + 1);
    W.flags = take(N * 8);
    W.scan[0] = take(N * 8);
    W.scan[1] = take(N * 8);
    W.temp_bytes = (int64_t)std::max(std::max(t_sort, t_scan), t_scan64);
    W.temp = take(W.temp_bytes);
    W.total = off;
    return ETF_OK;
}

int check_args(const etf_ctx *ctx, int64_t N)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->device < 0) return fail(ctx, ETF_ENOGPU, "host-only context");
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks: M and K are unknown");
    if (N <= 0) return fail(ctx, ETF_EINVAL, "N <= 0");
    if (N >= ((int64_t)1 << 31)) return fail(ctx, ETF_EINVAL, "N must be below 2^31");
    return ETF_OK;
}

int check_trees(const etf_ctx *ctx, int T, const int32_t *chunk_begin, std::vector<int32_t> &cb)
{
    const int M = ctx->M;
    if (T < 1 || T > M) return fail(ctx, ETF_EINVAL, "need 1 <= T <= M (T=%d, M=%d)", T, M);
    cb.resize(T + 1);
    if (chunk_begin) {
        for (int t = 0; t <= T; ++t) cb[t] = chunk_begin[t];
        if (cb[0] != 0 || cb[T] != M) return fail(ctx, ETF_EINVAL, "chunk_begin must run from 0 to M");
        for (int t = 0; t < T; ++t)
            if (cb[t + 1] <= cb[t]) return fail(ctx, ETF_EINVAL, "chunk_begin must be strictly increasing");
    } else {
        if (M % T != 0) return fail(ctx, ETF_EINVAL, "T=%d does not divide M=%d and no chunk_begin was given", T, M);
        for (int t = 0; t <= T; ++t) cb[t] = t * (M / T);
    }
    return ETF_OK;
}

// stable sort of (keys gathered through pos[cur]) with the positions as payload; flips cur
int sort_pass(etf_ctx *ctx, const BuildWs &W, char *ws, const uint8_t *rows, int M, const int32_t *ids_in, int64_t n, int c0,
              int c1, int &cur)
{
    hipStream_t st = (hipStream_t)ctx->stream;
    uint64_t *keys[2] = {(uint64_t *)(ws + W.keys[0]), (uint64_t *)(ws + W.keys[1])};
    uint32_t *pos[2] = {(uint32_t *)(ws + W.pos[0]), (uint32_t *)(ws + W.pos[1])};
    hipLaunchKernelGGL(k_build_keys, dim3(blocks(n)), dim3(BT), 0, st, rows, M, ids_in, pos[cur], n, c0, c1, keys[0]);
    HIP_TRY(ctx, hipGetLastError());
    const unsigned bits = c0 == c1 ? 32u : (unsigned)(8 * (c1 - c0));
    size_t tb = 0;
    HIP_TRY(ctx, rocprim::radix_sort_pairs(nullptr, tb, keys[0], keys[1], pos[cur], pos[cur ^ 1], (size_t)n, 0u, bits, st));
    if ((int64_t)tb > W.temp_bytes) return fail(ctx, ETF_ENOMEM, "radix sort scratch: %lld > %lld", (long long)tb, (long long)W.temp_bytes);
    tb = (size_t)W.temp_bytes;
    HIP_TRY(ctx, rocprim::radix_sort_pairs(ws + W.temp, tb, keys[0], keys[1], pos[cur], pos[cur ^ 1], (size_t)n, 0u, bits, st));
    cur ^= 1;
    return ETF_OK;
}

int build_impl(etf_ctx *ctx, const uint8_t *codes, int64_t N, const int32_t *ids, int T, const std::vector<int32_t> &cb,
               char *img, int64_t image_bytes, char *ws, const BuildWs &W)
{
    const int M = ctx->M, K = ctx->K;
    hipStream_t st = (hipStream_t)ctx->stream;
    HostIndex &ix = ctx->idx;
    ix.M = M; ix.K = K; ix.T = T; ix.N = N;
    ix.chunk_begin = cb;
    ix.device_built = true;
    ix.rstride0 = std::max(4, depth_class(cb[1] - cb[0]));
    ix.tree.assign(T, HostTree());
    for (int t = 0; t < T; ++t) {
        HostTree &tr = ix.tree[t];
        tr.c0 = cb[t];
        tr.D = cb[t + 1] - cb[t];
        tr.rstride = std::max(4, depth_class(tr.D));
        tr.level.assign(tr.D, HostLevel());
        tr.bucket.assign(tr.D, HostBucket());
        tr.nI.assign(tr.D, 0);
        tr.nL.assign(tr.D, 0);
        for (int l = 0; l < tr.D; ++l) {
            tr.bucket[l].width = tr.D - l;
            tr.bucket[l].stride = (tr.bucket[l].width + 3) & ~3;
        }
    }
    // The layout grows with the counts: arrays whose sizes are known keep their offsets when later counts arrive.
    const DevLayout &L = ctx->lay;
    auto fits = [&](int64_t upto, const char *what) -> int {
        if (upto > image_bytes) return fail(ctx, ETF_ENOMEM, "image buffer too small for %s: %lld > %lld", what, (long long)upto, (long long)image_bytes);
        return ETF_OK;
    };
    compute_layout(ctx);
    int rc = fits(L.ebegin, "the input codes and ids");   // codes, ids_in, ids_sorted end where ebegin starts
    if (rc) return rc;

    uint32_t *pos[2] = {(uint32_t *)(ws + W.pos[0]), (uint32_t *)(ws + W.pos[1])};
    uint32_t *head = (uint32_t *)(ws + W.head), *rank = (uint32_t *)(ws + W.rank), *scal = (uint32_t *)(ws + W.scal);
    uint8_t *d_codes = (uint8_t *)(img + L.codes);
    int32_t *d_ids_in = (int32_t *)(img + L.ids_in);

    // quantiser tables and the input codes
    auto put = [&](int64_t off, const std::vector<float> &v) {
        return v.empty() ? hipSuccess : hipMemcpyAsync(img + off, v.data(), v.size() * 4, hipMemcpyHostToDevice, st);
    };
    HIP_TRY(ctx, put(L.codebooks, ctx->codebooks));
    HIP_TRY(ctx, put(L.cb_centered, ctx->cb_centered));
    HIP_TRY(ctx, put(L.cb_norm, ctx->cb_norm));
    HIP_TRY(ctx, put(L.cb_mean, ctx->cb_mean));
    HIP_TRY(ctx, hipMemsetAsync(scal, 0, 16, st));
    const unsigned nb = blocks(N);
    ix.order.resize(M);
    BuildOrder ord;
    bool identity = true;
    for (int j = 0; j < ETF_MAX_M; ++j) {
        const int src = (j < M && !ctx->next_order.empty()) ? ctx->next_order[j] : j;
        if (j < M) ix.order[j] = src;
        ord.src[j] = (uint8_t)src;
        identity = identity && src == j;
    }
    if (identity) {
        if (d_codes != codes) HIP_TRY(ctx, hipMemcpyAsync(d_codes, codes, (size_t)N * M, hipMemcpyDeviceToDevice, st));
    } else {
        hipLaunchKernelGGL(k_build_permute, dim3(nb), dim3(BT), 0, st, codes, d_codes, N, M, ord);
        HIP_TRY(ctx, hipGetLastError());
    }
    hipLaunchKernelGGL(k_build_init, dim3(nb), dim3(BT), 0, st, d_codes, ids, N, M, K, pos[0], d_ids_in, scal);
    HIP_TRY(ctx, hipGetLastError());

    // (encoding, id) order by stable least-significant-part-first passes: id (only when ids are given: positions
    // ascend already), chunks 8.. (only when there are any), chunks 0..7
    int cur = 0;
    if (ids && (rc = sort_pass(ctx, W, ws, d_codes, M, d_ids_in, N, 0, 0, cur))) return rc;
    if (M > 8 && (rc = sort_pass(ctx, W, ws, d_codes, M, d_ids_in, N, 8, M, cur))) return rc;
    if ((rc = sort_pass(ctx, W, ws, d_codes, M, d_ids_in, N, 0, std::min(M, 8), cur))) return rc;
    const uint32_t *spos = pos[cur];

    hipLaunchKernelGGL(k_build_heads, dim3(nb), dim3(BT), 0, st, d_codes, spos, N, M, 0, M, head);
    HIP_TRY(ctx, hipGetLastError());
    {
        size_t tb = (size_t)W.temp_bytes;
        HIP_TRY(ctx, rocprim::inclusive_scan(ws + W.temp, tb, head, rank, (size_t)N, rocprim::plus<uint32_t>(), st));
    }
    // the counts read back from the device land in the context, not in this frame: a copy that is still pending when
    // an error path returns completes (at the caller's synchronisation) into memory that is still alive
    uint32_t *h_scal = ctx->build_scal;
    h_scal[0] = h_scal[1] = h_scal[2] = h_scal[3] = 0;
    HIP_TRY(ctx, hipMemcpyAsync(&h_scal[0], rank + (N - 1), 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipMemcpyAsync(&h_scal[2], scal + 2, 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    if (h_scal[2] & 1u) return fail(ctx, ETF_EINVAL, "a code byte is >= K=%d", K);
    if (h_scal[2] & 2u) return fail(ctx, ETF_EINVAL, "ids must be non-negative");
    const int64_t Nd = h_scal[0];
    if (Nd < 1 || Nd > N) return fail(ctx, ETF_EHIP, "device build returned %lld distinct encodings for %lld vectors", (long long)Nd, (long long)N);
    ix.Nd = Nd;
    ix.n_sample_enc = std::min(Nd, sample_size(ctx->opt, Nd));
    ix.n_sample_pos = std::min(N, sample_size(ctx->opt, N));
    compute_layout(ctx);
    rc = fits(L.tree[0].leaf_of >= 0 ? L.tree[0].leaf_of : L.tree[0].rec, "the sorted encodings");
    if (rc) return rc;

    uint32_t *d_ebegin = (uint32_t *)(img + L.ebegin);
    uint8_t *d_ecodes = (uint8_t *)(img + L.ecodes);
    hipLaunchKernelGGL(k_build_scatter, dim3(nb), dim3(BT), 0, st, d_codes, d_ids_in, spos, head, rank, N, M,
                       (int32_t *)(img + L.ids_sorted), (uint32_t *)(img + L.enc_of_pos), d_ebegin, d_ecodes, scal);
    HIP_TRY(ctx, hipGetLastError());
    hipLaunchKernelGGL(k_build_maxdup, dim3(nb), dim3(BT), 0, st, d_ebegin, scal);
    HIP_TRY(ctx, hipGetLastError());
    HIP_TRY(ctx, hipMemcpyAsync(&h_scal[1], scal + 1, 4, hipMemcpyDeviceToHost, st));  // read at the next synchronisation

    // threshold samples.  Tree modes: distinct encodings drawn through the vectors, repeats dropped (their number comes
    // back to the host: the sample's arrays and everything behind them are placed once it is known).
    const uint64_t seed = 0x1509051860ull ^ (uint64_t)N;
    {
        const int64_t S0 = ix.n_sample_enc;  // draws
        uint32_t *draw = head, *keep = rank, *kscan = (uint32_t *)(ws + W.keys[0]);  // free between the scatter above and the trees
        hipLaunchKernelGGL(k_build_sample_draw, dim3(blocks(S0)), dim3(BT), 0, st, d_ebegin, Nd, N, S0, seed, draw, keep);
        HIP_TRY(ctx, hipGetLastError());
        size_t tb = (size_t)W.temp_bytes;
        HIP_TRY(ctx, rocprim::inclusive_scan(ws + W.temp, tb, keep, kscan, (size_t)S0, rocprim::plus<uint32_t>(), st));
        HIP_TRY(ctx, hipMemcpyAsync(&h_scal[3], kscan + (S0 - 1), 4, hipMemcpyDeviceToHost, st));
        HIP_TRY(ctx, hipStreamSynchronize(st));
        const int64_t S_enc = h_scal[3];
        if (S_enc < 1 || S_enc > S0) return fail(ctx, ETF_EHIP, "device build: %lld of %lld sample draws kept", (long long)S_enc, (long long)S0);
        ix.n_sample_enc = S_enc;
        compute_layout(ctx);
        const uint64_t A = spread_multiplier(S_enc);
        hipLaunchKernelGGL(k_build_sample_place, dim3(blocks(S0)), dim3(BT), 0, st, draw, keep, kscan, S0, S_enc, inverse_mod(A, S_enc),
                           (uint64_t)(S_enc / 3), d_ecodes, M, (uint32_t *)(img + L.sample_enc), (uint8_t *)(img + L.sample_enc_codes));
        HIP_TRY(ctx, hipGetLastError());
    }
    // flat scan: input positions, one from each of S_pos strata
    const int64_t S_pos = ix.n_sample_pos;
    hipLaunchKernelGGL(k_build_sample, dim3(blocks(S_pos)), dim3(BT), 0, st, d_codes, N, M, S_pos, spread_multiplier(S_pos),
                       (uint64_t)(S_pos / 3), seed ^ 0x5DEECE66Dull, (uint32_t *)(img + L.sample_pos), (uint8_t *)(img + L.sample_pos_codes));
    HIP_TRY(ctx, hipGetLastError());
    hipLaunchKernelGGL(k_build_rec0, dim3(blocks(Nd)), dim3(BT), 0, st, d_ecodes, M, cb[1] - cb[0], Nd, (uint8_t *)(img + L.rec0),
                       ix.rstride0, depth_class(cb[1] - cb[0]) - (cb[1] - cb[0]));
    HIP_TRY(ctx, hipGetLastError());

    // ---- the trees
    uint8_t *lcp = (uint8_t *)(ws + W.lcp);
    uint64_t *flags = (uint64_t *)(ws + W.flags);
    uint64_t *scan[2] = {(uint64_t *)(ws + W.scan[0]), (uint64_t *)(ws + W.scan[1])};
    const unsigned nbd = blocks(Nd);
    for (int t = 0; t < T; ++t) {
        HostTree &tr = ix.tree[t];
        const int c0 = tr.c0, D = tr.D, pad = depth_class(D) - D;
        // the distinct encodings in the order of this tree's chunks (tree 0's are a prefix: sorted already)
        cur = 0;
        hipLaunchKernelGGL(k_build_iota, dim3(nbd), dim3(BT), 0, st, pos[0], Nd);
        HIP_TRY(ctx, hipGetLastError());
        if (t > 0) {
            if (D > 8 && (rc = sort_pass(ctx, W, ws, d_ecodes, M, nullptr, Nd, c0 + 8, c0 + D, cur))) return rc;
            if ((rc = sort_pass(ctx, W, ws, d_ecodes, M, nullptr, Nd, c0, c0 + std::min(D, 8), cur))) return rc;
        }
        const uint32_t *eord = pos[cur];
        hipLaunchKernelGGL(k_build_heads, dim3(nbd), dim3(BT), 0, st, d_ecodes, eord, Nd, M, c0, D, head);
        HIP_TRY(ctx, hipGetLastError());
        {
            size_t tb = (size_t)W.temp_bytes;
            HIP_TRY(ctx, rocprim::inclusive_scan(ws + W.temp, tb, head, rank, (size_t)Nd, rocprim::plus<uint32_t>(), st));
        }
        uint32_t h_U = 0;
        HIP_TRY(ctx, hipMemcpyAsync(&h_U, rank + (Nd - 1), 4, hipMemcpyDeviceToHost, st));
        HIP_TRY(ctx, hipStreamSynchronize(st));
        const int64_t U = h_U;
        if (U < 1 || U > Nd || (T == 1 && U != Nd)) return fail(ctx, ETF_EHIP, "device build: tree %d has %lld leaves for %lld encodings", t, (long long)U, (long long)Nd);
        tr.U = U;
        compute_layout(ctx);
        const DevTreeLayout TL = L.tree[t];
        rc = fits(TL.icode[0], "a tree's records");   // leaf_of and rec end where the first level starts
        if (rc) return rc;
        uint8_t *rec = (uint8_t *)(img + TL.rec);
        hipLaunchKernelGGL(k_tree_records, dim3(nbd), dim3(BT), 0, st, d_ecodes, M, c0, D, eord, head, rank, Nd,
                           TL.leaf_of >= 0 ? (uint32_t *)(img + TL.leaf_of) : nullptr, rec, tr.rstride, pad);
        HIP_TRY(ctx, hipGetLastError());
        hipLaunchKernelGGL(k_tree_lcp, dim3(blocks(U + 1)), dim3(BT), 0, st, rec, tr.rstride, pad, D, U, lcp);
        HIP_TRY(ctx, hipGetLastError());
        const unsigned nbu = blocks(U);
        int sc = 0;
        for (int l = 1; l <= D; ++l) {
            hipLaunchKernelGGL(k_tree_flags, dim3(nbu), dim3(BT), 0, st, lcp, U, l, D, flags);
            HIP_TRY(ctx, hipGetLastError());
            size_t tb = (size_t)W.temp_bytes;
            HIP_TRY(ctx, rocprim::inclusive_scan(ws + W.temp, tb, flags, scan[sc], (size_t)U, rocprim::plus<uint64_t>(), st));
            uint64_t tot = 0;
            HIP_TRY(ctx, hipMemcpyAsync(&tot, scan[sc] + (U - 1), 8, hipMemcpyDeviceToHost, st));
            HIP_TRY(ctx, hipStreamSynchronize(st));
            tr.nI[l - 1] = (int64_t)(tot & 0xFFFFFFFFu);
            tr.nL[l - 1] = (int64_t)(tot >> 32);
            compute_layout(ctx);
            const DevTreeLayout TL2 = L.tree[t];
            rc = fits(TL2.lrow[l - 1] + tr.nL[l - 1] * 4, "a tree level");
            if (rc) return rc;
            hipLaunchKernelGGL(k_tree_level, dim3(nbu), dim3(BT), 0, st, rec, tr.rstride, pad, D, lcp, scan[sc], scan[sc ^ 1], U, l,
                               (uint8_t *)(img + TL2.icode[l - 1]), (uint32_t *)(img + TL2.iparent[l - 1]),
                               (uint8_t *)(img + TL2.lcodes[l - 1]), tr.bucket[l - 1].stride,
                               (uint32_t *)(img + TL2.lparent[l - 1]), (uint32_t *)(img + TL2.lrow[l - 1]));
            HIP_TRY(ctx, hipGetLastError());
            sc ^= 1;
        }
        int64_t leaves = 0;
        for (int l = 0; l < D; ++l) leaves += tr.nL[l];
        if (leaves != U) return fail(ctx, ETF_EHIP, "device build: tree %d has %lld leaves in its levels, %lld sub-encodings", t, (long long)leaves, (long long)U);
    }
    HIP_TRY(ctx, hipStreamSynchronize(st));
    compute_layout(ctx);
    rc = fits(L.total, "the index");
    if (rc) return rc;
    ix.max_dup = h_scal[1];
    if (ix.max_dup < 1) return fail(ctx, ETF_EHIP, "device build: no id range");
    ix.built = true;
    ctx->dev_base = img;
    return ETF_OK;
}

}  // namespace

extern "C" int etf_index_build_device_bytes(const etf_ctx *ctx, int64_t N, int T, const int32_t *chunk_begin,
                                            int64_t *image_bytes, int64_t *workspace_bytes)
{
    int rc = check_args(ctx, N);
    if (rc) return rc;
    if (!image_bytes || !workspace_bytes) return fail(ctx, ETF_EINVAL, "output pointer is null");
    std::vector<int32_t> cb;
    rc = check_trees(ctx, T, chunk_begin, cb);
    if (rc) return rc;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    BuildWs W;
    rc = plan_ws(ctx, N, W);
    if (rc) return rc;
    *image_bytes = image_bytes_bound(ctx, N, T, cb.data());
    *workspace_bytes = W.total;
    return ETF_OK;
}

extern "C" int etf_index_build_device(etf_ctx *ctx, const uint8_t *codes, int64_t N, const int32_t *ids, int T,
                                      const int32_t *chunk_begin, void *image, int64_t image_bytes, void *workspace,
                                      int64_t workspace_bytes)
{
    int rc = check_args(ctx, N);
    if (rc) return rc;
    if (!codes) return fail(ctx, ETF_EINVAL, "codes is null");
    std::vector<int32_t> cb;
    rc = check_trees(ctx, T, chunk_begin, cb);
    if (rc) return rc;
    if (!ctx->next_term.empty()) return fail(ctx, ETF_ESTATE, "a leaf payload is pending: indexes with leaf terms are built by etf_index_build");
    if (!image || !workspace) return fail(ctx, ETF_EINVAL, "image or workspace is null");
    if ((((uintptr_t)image | (uintptr_t)workspace) & 255) != 0) return fail(ctx, ETF_EINVAL, "image and workspace must be 256-byte aligned");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    BuildWs W;
    rc = plan_ws(ctx, N, W);
    if (rc) return rc;
    if (workspace_bytes < W.total) return fail(ctx, ETF_ENOMEM, "workspace too small: %lld < %lld", (long long)workspace_bytes, (long long)W.total);
    drop_index(ctx);
    rc = build_impl(ctx, codes, N, ids, T, cb, (char *)image, image_bytes, (char *)workspace, W);
    if (rc) {
        (void)hipStreamSynchronize((hipStream_t)ctx->stream);  // nothing of a failed build may still be running in the buffers
        drop_index(ctx);
    }
    return rc;
}
