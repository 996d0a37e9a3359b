// Index build on the device (Algorithm 1's first half; Section 3.2's remark on building in parallel): the
// lexicographic sort of the encodings, the merge of repeated encodings into id ranges, and the threshold samples.
// The sort and the prefix sum are rocPRIM's device-wide radix sort and scan; everything around them is kernels of
// this file.  The image written here holds what the LDS-resident kernels, the flat scan and the exact kernel read:
// no per-tree level arrays (those kernels take an encoding's shared prefix from its sorted neighbour instead).
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

// Sort key of the vector at position pos[i].  part 0: its id; part 1: chunks 8.. of its encoding; part 2: chunks
// 0..7.  Chunks go most significant first, so that integer order is lexicographic order; a part of n chunks
// fills the low 8 n bits (the sort then leaves out the empty high bits).
__global__ void __launch_bounds__(BT) k_build_keys(const uint8_t *codes, const int32_t *ids_in, const uint32_t *pos,
                                                   int64_t N, int M, int part, uint64_t *keys)
{
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i >= N) return;
    const int64_t p = pos[i];
    uint64_t k = 0;
    if (part == 0) {
        k = (uint64_t)(uint32_t)ids_in[p];
    } else {
        const int c0 = part == 1 ? 8 : 0, c1 = part == 1 ? M : min(M, 8);
        for (int c = c0; c < c1; ++c) k |= (uint64_t)codes[p * M + c] << (8 * (c1 - 1 - c));
    }
    keys[i] = k;
}

// head[i] = 1 where the i-th vector in sorted order starts a new encoding
__global__ void __launch_bounds__(BT) k_build_heads(const uint8_t *codes, const uint32_t *pos, int64_t N, int M, uint32_t *head)
{
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i >= N) return;
    uint32_t h = 1;
    if (i > 0) {
        const uint8_t *a = codes + (int64_t)pos[i] * M, *b = codes + (int64_t)pos[i - 1] * M;
        h = 0;
        for (int m = 0; m < M; ++m) h |= a[m] != b[m];
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
    if ((threadIdx.x & 63) == 0 && n) atomicMax(&scal[1], n);
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
// with them the sample groups the kernels cut the sample into) hold rows from all over the range, never a run of
// neighbouring encodings.
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

// multiplier of the slot -> stratum map: near S / golden ratio, coprime to S
uint64_t spread_multiplier(int64_t S)
{
    if (S <= 2) return 1;
    int64_t a = (int64_t)((double)S * 0.6180339887498949);
    a = std::max<int64_t>(1, std::min(a, S - 1));
    while (std::gcd(a, S) != 1) ++a;  // S - 1 is coprime to S: the loop ends below S
    return (uint64_t)a;
}

struct BuildWs {
    int64_t keys[2], pos[2], head, rank, scal, temp, temp_bytes, total;
};

int plan_ws(const etf_ctx *ctx, int64_t N, BuildWs &W)
{
    size_t t_sort = 0, t_scan = 0;
    // size queries: no launch, no device memory touched
    hipError_t e = rocprim::radix_sort_pairs(nullptr, t_sort, (uint64_t *)nullptr, (uint64_t *)nullptr, (uint32_t *)nullptr,
                                             (uint32_t *)nullptr, (size_t)N, 0u, 64u, (hipStream_t)ctx->stream);
    if (e != hipSuccess) return fail(ctx, ETF_EHIP, "radix sort size query: %s", hipGetErrorString(e));
    e = rocprim::inclusive_scan(nullptr, t_scan, (uint32_t *)nullptr, (uint32_t *)nullptr, (size_t)N, rocprim::plus<uint32_t>(),
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
    W.temp_bytes = (int64_t)std::max(t_sort, t_scan);
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

}  // namespace

extern "C" int etf_index_build_device_bytes(const etf_ctx *ctx, int64_t N, int64_t *image_bytes, int64_t *workspace_bytes)
{
    int rc = check_args(ctx, N);
    if (rc) return rc;
    if (!image_bytes || !workspace_bytes) return fail(ctx, ETF_EINVAL, "output pointer is null");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    DevLayout L;
    lean_layout(ctx, N, L);
    BuildWs W;
    rc = plan_ws(ctx, N, W);
    if (rc) return rc;
    *image_bytes = L.total;
    *workspace_bytes = W.total;
    return ETF_OK;
}

extern "C" int etf_index_build_device(etf_ctx *ctx, const uint8_t *codes, int64_t N, const int32_t *ids, int T,
                                      const int32_t *chunk_begin, void *image, int64_t image_bytes, void *workspace,
                                      int64_t workspace_bytes)
{
    int rc = check_args(ctx, N);
    if (rc) return rc;
    const int M = ctx->M, K = ctx->K;
    if (!codes) return fail(ctx, ETF_EINVAL, "codes is null");
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
    if (!image || !workspace) return fail(ctx, ETF_EINVAL, "image or workspace is null");
    if ((((uintptr_t)image | (uintptr_t)workspace) & 255) != 0) return fail(ctx, ETF_EINVAL, "image and workspace must be 256-byte aligned");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    DevLayout L;
    lean_layout(ctx, N, L);
    BuildWs W;
    rc = plan_ws(ctx, N, W);
    if (rc) return rc;
    if (image_bytes < L.total) return fail(ctx, ETF_ENOMEM, "image buffer too small: %lld < %lld", (long long)image_bytes, (long long)L.total);
    if (workspace_bytes < W.total) return fail(ctx, ETF_ENOMEM, "workspace too small: %lld < %lld", (long long)workspace_bytes, (long long)W.total);

    drop_index(ctx);
    hipStream_t st = (hipStream_t)ctx->stream;
    char *img = (char *)image, *ws = (char *)workspace;
    uint64_t *keys[2] = {(uint64_t *)(ws + W.keys[0]), (uint64_t *)(ws + W.keys[1])};
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
    if (d_codes != codes) HIP_TRY(ctx, hipMemcpyAsync(d_codes, codes, (size_t)N * M, hipMemcpyDeviceToDevice, st));
    HIP_TRY(ctx, hipMemsetAsync(scal, 0, 16, st));

    const unsigned nb = blocks(N);
    hipLaunchKernelGGL(k_build_init, dim3(nb), dim3(BT), 0, st, d_codes, ids, N, M, K, pos[0], d_ids_in, scal);
    HIP_TRY(ctx, hipGetLastError());

    // (encoding, id) order by stable least-significant-part-first passes: id (only when ids are given: positions
    // ascend already), chunks 8.. (only when there are any), chunks 0..7
    int cur = 0;
    for (int part = ids ? 0 : 1; part <= 2; ++part) {
        if (part == 1 && M <= 8) continue;
        const int nchunks = part == 1 ? M - 8 : std::min(M, 8);
        const unsigned b0 = 0u, b1 = part == 0 ? 32u : (unsigned)(8 * nchunks);
        hipLaunchKernelGGL(k_build_keys, dim3(nb), dim3(BT), 0, st, d_codes, d_ids_in, pos[cur], N, M, part, keys[0]);
        HIP_TRY(ctx, hipGetLastError());
        size_t tb = 0;
        HIP_TRY(ctx, rocprim::radix_sort_pairs(nullptr, tb, keys[0], keys[1], pos[cur], pos[cur ^ 1], (size_t)N, b0, b1, st));
        if ((int64_t)tb > W.temp_bytes) return fail(ctx, ETF_ENOMEM, "radix sort scratch: %lld > %lld", (long long)tb, (long long)W.temp_bytes);
        tb = (size_t)W.temp_bytes;
        HIP_TRY(ctx, rocprim::radix_sort_pairs(ws + W.temp, tb, keys[0], keys[1], pos[cur], pos[cur ^ 1], (size_t)N, b0, b1, st));
        cur ^= 1;
    }
    const uint32_t *spos = pos[cur];

    hipLaunchKernelGGL(k_build_heads, dim3(nb), dim3(BT), 0, st, d_codes, spos, N, M, head);
    HIP_TRY(ctx, hipGetLastError());
    {
        size_t tb = (size_t)W.temp_bytes;
        HIP_TRY(ctx, rocprim::inclusive_scan(ws + W.temp, tb, head, rank, (size_t)N, rocprim::plus<uint32_t>(), st));
    }
    uint32_t *d_ebegin = (uint32_t *)(img + L.ebegin);
    uint8_t *d_ecodes = (uint8_t *)(img + L.ecodes);
    hipLaunchKernelGGL(k_build_scatter, dim3(nb), dim3(BT), 0, st, d_codes, d_ids_in, spos, head, rank, N, M,
                       (int32_t *)(img + L.ids_sorted), (uint32_t *)(img + L.enc_of_pos), d_ebegin, d_ecodes, scal);
    HIP_TRY(ctx, hipGetLastError());
    hipLaunchKernelGGL(k_build_maxdup, dim3(nb), dim3(BT), 0, st, d_ebegin, scal);
    HIP_TRY(ctx, hipGetLastError());

    uint32_t h_scal[4] = {0, 0, 0, 0};
    HIP_TRY(ctx, hipMemcpyAsync(h_scal, scal, 16, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    if (h_scal[2] & 1u) return fail(ctx, ETF_EINVAL, "a code byte is >= K=%d", K);
    if (h_scal[2] & 2u) return fail(ctx, ETF_EINVAL, "ids must be non-negative");
    const int64_t Nd = h_scal[0], max_dup = h_scal[1];
    if (Nd < 1 || Nd > N || max_dup < 1) return fail(ctx, ETF_EHIP, "device build returned %lld distinct encodings for %lld vectors", (long long)Nd, (long long)N);

    // threshold samples (of the distinct encodings for the tree modes, of the input positions for the flat scan)
    const int64_t S_enc = std::min(Nd, sample_size(ctx->opt, Nd)), S_pos = std::min(N, sample_size(ctx->opt, N));
    const uint64_t seed = 0x1509051860ull ^ (uint64_t)N;
    hipLaunchKernelGGL(k_build_sample, dim3(blocks(S_enc)), dim3(BT), 0, st, d_ecodes, Nd, M, S_enc, spread_multiplier(S_enc),
                       (uint64_t)(S_enc / 3), seed, (uint32_t *)(img + L.sample_enc), (uint8_t *)(img + L.sample_enc_codes));
    HIP_TRY(ctx, hipGetLastError());
    hipLaunchKernelGGL(k_build_sample, dim3(blocks(S_pos)), dim3(BT), 0, st, d_codes, N, M, S_pos, spread_multiplier(S_pos),
                       (uint64_t)(S_pos / 3), seed ^ 0x5DEECE66Dull, (uint32_t *)(img + L.sample_pos), (uint8_t *)(img + L.sample_pos_codes));
    HIP_TRY(ctx, hipGetLastError());
    HIP_TRY(ctx, hipStreamSynchronize(st));

    HostIndex &ix = ctx->idx;
    ix.M = M; ix.K = K; ix.T = T; ix.N = N; ix.Nd = Nd; ix.max_dup = max_dup;
    ix.chunk_begin = cb;
    ix.n_sample_enc = S_enc;
    ix.n_sample_pos = S_pos;
    ix.tree.assign(T, HostTree());
    for (int t = 0; t < T; ++t) {
        ix.tree[t].c0 = cb[t];
        ix.tree[t].D = cb[t + 1] - cb[t];
    }
    ix.lean = true;
    ix.built = true;
    L.tree.assign(T, DevTreeLayout());
    ctx->lay = L;
    ctx->dev_base = img;
    return ETF_OK;
}
