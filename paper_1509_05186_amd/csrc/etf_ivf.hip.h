// IVFADC on the merged, sorted encodings (paper, "Application on related algorithms", Table 1: a coarse quantiser of
// K' cells, w probed inverted lists per query, residuals product-quantised; the ADC part of every probed list is
// what the Encoding Tree replaces).  Included at the end of etf_device.hip (uses its launch helpers).
//
// A stored vector is (cell, encoding of x - centroid[cell]); its distance to a query q splits into
//     ||q - c - r||^2  =  ||q - c||^2  +  (||r||^2 + 2 <c, r>)  -  2 <q, r>
// with c the centroid and r the reconstructed residual: the first term is one number per (query, probed cell) and
// comes from the probe selection, the second is a constant of the entry stored beside its encoding (the paper's
// "extra information stored on the leaf", Experiments section), the third is a sum of M entries of scalar-product
// tables <q_m, codeword> that depend on the query alone and are shared by all cells.  So no table is built per
// (query, cell).  Entries are sorted by (cell, encoding): list j is a contiguous range, equal encodings inside a
// cell are one entry with an id range (one leaf), exactly the leaf sequence of the list's Encoding Tree.
#pragma once

namespace etf {

// ------------------------------------------------------------------------------------------------
// Squared distances between vectors and centroids in float32, every one the sum of its (x - c)^2 terms in dimension
// order with one rounding per operation and nothing fused: the rule under which the cell of a vector and the probed
// cells of a query are decided, so that a float32 reference reproduces every decision.
//     thread = vector; a block of 256 vectors walks the centroids 32 at a time (partial sums in registers) and the
//     dimensions 32 at a time (both operands staged in LDS: xs[j][thread], cs[j][centroid]).
//     ARGMIN: best[n] = nearest centroid, lowest index on ties.  Otherwise dist[n][Kc] is written, and the centroids
//     are cut into gridDim.y slices of cslice (a multiple of 32), one per workgroup row: few vectors (a batch of
//     queries) still fill the chip.
//     grid (ceil(n / 256), slices), block 256.
// ------------------------------------------------------------------------------------------------
template <bool ARGMIN>
__global__ __launch_bounds__(256) void k_ivf_coarse(const float *__restrict__ x, int64_t n, int d, const float *__restrict__ cent,
                                                    int Kc, float *__restrict__ dist, int32_t *__restrict__ best, int cslice)
{
    constexpr int CT = 32, DJ = 32;
    __shared__ float xs[DJ][257];  // rows one float longer than the block: the transposing stores below hit 32 banks, not 1
    __shared__ float cs[DJ][CT];
    const int t = threadIdx.x;
    const int64_t v0 = (int64_t)blockIdx.x * 256, v = v0 + t;
    float bestd = 3.402823466e+38f;
    int besti = 0;
    const int cbeg = ARGMIN ? 0 : (int)blockIdx.y * cslice, cend = ARGMIN ? Kc : min(Kc, cbeg + cslice);
    for (int c0 = cbeg; c0 < cend; c0 += CT) {
        float acc[CT];
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[c] = 0.f;
        for (int j0 = 0; j0 < d; j0 += DJ) {
            __syncthreads();
            // stage 256 vectors x 32 dimensions (coalesced along the dimension, transposed into LDS) and 32 centroids
            for (int i = t; i < 256 * DJ; i += 256) {
                const int vv = i / DJ, j = i % DJ;
                xs[j][vv] = (v0 + vv < n && j0 + j < d) ? x[(v0 + vv) * d + j0 + j] : 0.f;
            }
            for (int i = t; i < CT * DJ; i += 256) {
                const int c = i % CT, j = i / CT;  // consecutive lanes: consecutive words of a row of cs
                cs[j][c] = (c0 + c < Kc && j0 + j < d) ? cent[(int64_t)(c0 + c) * d + j0 + j] : 0.f;
            }
            __syncthreads();
            const int nj = min(DJ, d - j0);
            for (int j = 0; j < nj; ++j) {
                const float xj = xs[j][t];
                {
#pragma clang fp contract(off)
#pragma unroll
                    for (int c = 0; c < CT; ++c) {
                        const float df = xj - cs[j][c];
                        const float p = df * df;
                        acc[c] = acc[c] + p;
                    }
                }
            }
        }
        if (ARGMIN) {
#pragma unroll
            for (int c = 0; c < CT; ++c)
                if (c0 + c < Kc && acc[c] < bestd) {
                    bestd = acc[c];
                    besti = c0 + c;
                }
        } else if (v < n) {
#pragma unroll
            for (int c = 0; c < CT; ++c)
                if (c0 + c < Kc) dist[v * Kc + c0 + c] = acc[c];
        }
    }
    if (ARGMIN && v < n) best[v] = besti;
}

// r[n][d] = x[n][d] - centroid[cell[n]][d], one float32 subtraction per component
__global__ __launch_bounds__(256) void k_ivf_residual(const float *__restrict__ x, int64_t n, int d, const float *__restrict__ cent,
                                                      const int32_t *__restrict__ cell, float *__restrict__ r)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n * d) return;
    const int64_t v = i / d;
    const int j = (int)(i - v * d);
    r[i] = x[i] - cent[(int64_t)cell[v] * d + j];
}

// ------------------------------------------------------------------------------------------------
// Probe selection: the w cells with the smallest (distance, index) of one query, ascending.  A radix select on the
// float bits of the distances over the query's row of the distance matrix (and one on the cell numbers among exact
// ties at the w-th, if they matter), then the w keys at or below the w-th are collected and sorted.
//     grid (queries), block 256, dynamic LDS 8 * pow2(w) bytes; Kc <= 65536.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_ivf_probe(const float *__restrict__ dist, int Kc, int w, int32_t *__restrict__ probes)
{
    extern __shared__ uint64_t pk[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_n;
    const int64_t q = blockIdx.x;
    const float *row = dist + q * Kc;
    // the w-th smallest distance, then, if more cells tie with it than are still needed, the largest cell number to take
    __shared__ uint32_t sel_sh[8];
    uint32_t vstar, rank_in_ties, n_ties, cstar = 0xFFFFFFFFu;
    block_radix_select(
        Kc, (uint32_t)min(w, Kc), [&](int c, uint32_t &v) { v = __float_as_uint(row[c]); return true; }, hist, sel_sh, vstar,
        rank_in_ties, n_ties);
    if (n_ties > rank_in_ties) {
        uint32_t r2, n2;
        block_radix_select(
            Kc, rank_in_ties,
            [&](int c, uint32_t &v) {
                if (__float_as_uint(row[c]) != vstar) return false;
                v = (uint32_t)c;
                return true;
            },
            hist, sel_sh, cstar, r2, n2);
    }
    if (threadIdx.x == 0) s_n = 0;
    __syncthreads();
    for (int c = threadIdx.x; c < Kc; c += 256) {
        const uint32_t v = __float_as_uint(row[c]);
        if (v < vstar || (v == vstar && (uint32_t)c <= cstar)) {
            const uint32_t pos = atomicAdd(&s_n, 1u);
            if (pos < (uint32_t)w) pk[pos] = ((uint64_t)v << 16) | (uint32_t)c;
        }
    }
    __syncthreads();
    const int w2 = pow2_at_least(w);
    for (int i = w + threadIdx.x; i < w2; i += 256) pk[i] = ~0ull;
    __syncthreads();
    bitonic_sort_u64(pk, w2);
    for (int i = threadIdx.x; i < w; i += 256) probes[q * w + i] = (int32_t)(pk[i] & 0xFFFFu);
}

// ------------------------------------------------------------------------------------------------
// The probed lists of one query.
// ------------------------------------------------------------------------------------------------
struct IvfScanArgs {
    const float *lut;         // [nq][M][K] scalar products <q_m, codeword>
    const float *coarse;      // [nq][Kc] squared distances to the centroids
    const int32_t *probes;    // [nq][w]
    int M, K, Kc, w, k;
    const uint32_t *lbegin;   // [Kc+1]
    const uint8_t *ecodes;    // [Ne][M]
    const float *eterm;       // [Ne]
    const uint32_t *ebegin;   // [Ne+1]
    const int32_t *ids;       // [N] ids sorted by (cell, encoding, id)
    uint32_t *cnt;            // [nq]
    uint64_t *cand;           // [nq][C]
    uint32_t C;
    uint32_t *flag;           // [nq]
    uint32_t *nflag;          // running count of queries answered by the exact kernel
    int32_t *out_ids;         // [nq][k]   (exact kernel)
    float *out_dist;          // [nq][k]
};

// distance of one entry: tab = the query's tables in LDS, bt = ||q - c||^2 + the entry's constant term.
// The three terms cancel when the query is close to the stored vector; what is left is never reported below zero.
__device__ __forceinline__ float ivf_distance(const float *tab, const uint8_t *__restrict__ c, int M, int K, float bt)
{
    float s = 0.f;
    for (int m = 0; m < M; ++m) s += tab[m * K + c[m]];
    return fmaxf(fmaf(-2.f, s, bt), 0.f);
}

// The same distance from the code bytes packed into words (c[m] = byte m & 3 of word m >> 2): the entries' codes
// are fetched with one 8- or 16-byte load where M allows it.  Same additions in the same order as ivf_distance.
__device__ __forceinline__ void ivf_load_codes(const uint8_t *__restrict__ c, int M, uint32_t (&w)[4])
{
    w[0] = w[1] = w[2] = w[3] = 0u;
    if (M == 8) {
        const uint2 v = *reinterpret_cast<const uint2 *>(c);
        w[0] = v.x;
        w[1] = v.y;
    } else if (M == 16) {
        const uint4 v = *reinterpret_cast<const uint4 *>(c);
        w[0] = v.x;
        w[1] = v.y;
        w[2] = v.z;
        w[3] = v.w;
    } else {
        for (int m = 0; m < M; ++m) w[m >> 2] |= (uint32_t)c[m] << (8 * (m & 3));
    }
}
__device__ __forceinline__ float ivf_distance_words(const float *tab, const uint32_t (&w)[4], int M, int K, float bt)
{
    float s = 0.f;
#pragma unroll
    for (int m = 0; m < 16; ++m)
        if (m < M) s += tab[m * K + ((w[m >> 2] >> (8 * (m & 3))) & 255u)];
    return fmaxf(fmaf(-2.f, s, bt), 0.f);
}

// Every entry of the probed lists once: wave v of the workgroup takes lists v, v + 4, ..., its lanes the entries of a
// list 128 at a time, two per lane, so that the loads of two entries (codes, stored term) are in flight together
// and no position has to be looked up among the lists.  f(entry, distance) runs for every entry.
// CM, CK: M and K as constants (the common shape, loops unrolled and table offsets immediate), or 0: taken from a.
template <int CM, int CK, class F>
__device__ __forceinline__ void ivf_walk_shape(const IvfScanArgs &a, const float *tab, const uint32_t *s_off, const uint32_t *s_lo,
                                               const float *s_base, F f)
{
    const int M = CM ? CM : a.M, K = CK ? CK : a.K;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    for (int p = wave; p < a.w; p += nw) {
        const uint32_t lo = s_lo[p], n = s_off[p + 1] - s_off[p];
        const float base = s_base[p];
        for (uint32_t i0 = lane; i0 < n; i0 += 128) {
            const bool two = i0 + 64 < n;
            const uint32_t e0 = lo + i0, e1 = two ? e0 + 64 : e0;
            uint32_t w0[4], w1[4];
            ivf_load_codes(a.ecodes + (int64_t)e0 * M, M, w0);
            ivf_load_codes(a.ecodes + (int64_t)e1 * M, M, w1);
            const float t0 = a.eterm[e0], t1 = a.eterm[e1];
            const float d0 = ivf_distance_words(tab, w0, M, K, base + t0);
            const float d1 = ivf_distance_words(tab, w1, M, K, base + t1);
            f(e0, d0);
            if (two) f(e1, d1);
        }
    }
}

template <class F>
__device__ __forceinline__ void ivf_walk(const IvfScanArgs &a, const float *tab, const uint32_t *s_off, const uint32_t *s_lo,
                                         const float *s_base, F f)
{
    if (a.M == 8 && a.K == 256)
        ivf_walk_shape<8, 256>(a, tab, s_off, s_lo, s_base, f);
    else
        ivf_walk_shape<0, 0>(a, tab, s_off, s_lo, s_base, f);
}

// The w probed lists of a query as one sequence of entries: s_off[p] = entries before list p.  Thread i of a flat
// position finds its list by bisection.
struct IvfLists {
    const uint32_t *s_off;   // [w+1] LDS
    const uint32_t *s_lo;    // [w]   LDS: first entry of list p
    const float *s_base;     // [w]   LDS: ||q - centroid||^2 of list p
    int w;
    __device__ __forceinline__ int list_of(uint32_t i) const
    {
        int lo = 0, hi = w - 1;  // largest p with s_off[p] <= i
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (s_off[mid] <= i) lo = mid;
            else hi = mid - 1;
        }
        return lo;
    }
};

__device__ __forceinline__ void ivf_setup_lists(const IvfScanArgs &a, int64_t q, uint32_t *s_off, uint32_t *s_lo, float *s_base)
{
    // list lengths, then their running sum (w is small: one thread adds them up)
    for (int p = threadIdx.x; p < a.w; p += blockDim.x) {
        const int cell = a.probes[q * a.w + p];
        s_lo[p] = a.lbegin[cell];
        s_off[p + 1] = a.lbegin[cell + 1] - a.lbegin[cell];
        s_base[p] = a.coarse[q * a.Kc + cell];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        s_off[0] = 0;
        for (int p = 0; p < a.w; ++p) {
            run += s_off[p + 1];
            s_off[p + 1] = run;
        }
    }
    __syncthreads();
}

// bytes of dynamic LDS of the two kernels below: tables, list bookkeeping, (scan only) the histogram
constexpr int IVF_HIST_BITS = 12;  // sign-free float bits >> 19: exponent and four mantissa bits (bins 6 % wide)
__host__ __device__ inline size_t ivf_lds_bytes(int M, int K, int w, bool hist)
{
    return (size_t)M * K * 4 + (size_t)(3 * w + 4) * 4 + (hist ? ((size_t)4 << IVF_HIST_BITS) : 0);
}

// ------------------------------------------------------------------------------------------------
// Scan of the probed lists of one query: every entry's distance from the query's tables in LDS (lane = entry).
//     Pass 1 counts the vectors per distance bin (a histogram over the upper bits of the float) and finds the bin in
//     which the running count reaches k: its upper edge bounds the k-th distance.  Pass 2 evaluates the entries again
//     and appends those at or below the bound to the query's candidate list, which k_select orders and expands.
//     grid (queries), block 256, dynamic LDS ivf_lds_bytes(..., true).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_ivf_scan(IvfScanArgs a)
{
    extern __shared__ float ivf_lds[];
    float *tab = ivf_lds;
    uint32_t *s_off = reinterpret_cast<uint32_t *>(tab + a.M * a.K);
    uint32_t *s_lo = s_off + a.w + 2;
    float *s_base = reinterpret_cast<float *>(s_lo + a.w + 1);
    uint32_t *hist = reinterpret_cast<uint32_t *>(s_base + a.w + 1);
    __shared__ uint32_t s_part[256];
    __shared__ uint32_t s_tau, s_cnt;
    constexpr int NB = 1 << IVF_HIST_BITS, SH = 31 - IVF_HIST_BITS;
    const int64_t q = blockIdx.x;
    for (int i = threadIdx.x; i < a.M * a.K; i += 256) tab[i] = a.lut[q * a.M * a.K + i];
    for (int i = threadIdx.x; i < NB; i += 256) hist[i] = 0;
    if (threadIdx.x == 0) s_cnt = 0;
    ivf_setup_lists(a, q, s_off, s_lo, s_base);
    ivf_walk(a, tab, s_off, s_lo, s_base, [&](uint32_t e, float d) {
        atomicAdd(&hist[__float_as_uint(d) >> SH], min(a.ebegin[e + 1] - a.ebegin[e], (uint32_t)a.k));
    });
    __syncthreads();
    // the bin in which the running count of vectors reaches k (thread t owns bins [t * NB/256, (t+1) * NB/256))
    {
        constexpr int PER = NB / 256;
        uint32_t part = 0;
        for (int b = 0; b < PER; ++b) part += hist[threadIdx.x * PER + b];
        s_part[threadIdx.x] = part;
        if (threadIdx.x == 0) s_tau = 0x7F800000u;  // fewer than k vectors in the probed lists: everything passes
        __syncthreads();
        uint32_t below = 0;
        for (int t2 = 0; t2 < (int)threadIdx.x; ++t2) below += s_part[t2];
        if (below < (uint32_t)a.k && below + part >= (uint32_t)a.k) {
            int b = 0;
            for (; b < PER - 1; ++b) {
                const uint32_t h = hist[threadIdx.x * PER + b];
                if (below + h >= (uint32_t)a.k) break;
                below += h;
            }
            s_tau = (((uint32_t)(threadIdx.x * PER + b) + 1u) << SH) - 1u;  // upper edge of that bin
        }
        __syncthreads();
    }
    const uint32_t tau = s_tau;
    ivf_walk(a, tab, s_off, s_lo, s_base, [&](uint32_t e, float d) {
        const uint32_t bits = __float_as_uint(d);
        if (bits <= tau) {
            const uint32_t pos = atomicAdd(&s_cnt, 1u);
            if (pos < a.C) a.cand[q * a.C + pos] = ((uint64_t)bits << 32) | e;
        }
    });
    __syncthreads();
    if (threadIdx.x == 0) a.cnt[q] = s_cnt;
}

// ------------------------------------------------------------------------------------------------
// Exact selection over the probed lists of one query, without any buffer that depends on the data (candidate
// overflow, huge groups of exactly equal distances): the radix select of k_exact on the 64-bit key (distance bits,
// id), every pass evaluating the entries again with the same arithmetic as the scan.  A query whose probed lists
// hold fewer than k vectors gets id -1 and +inf beyond them.
//     grid (queries), block 256, dynamic LDS ivf_lds_bytes(..., false); only flagged queries do any work.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_ivf_exact(IvfScanArgs a)
{
    extern __shared__ float ivf_lds[];
    float *tab = ivf_lds;
    uint32_t *s_off = reinterpret_cast<uint32_t *>(tab + a.M * a.K);
    uint32_t *s_lo = s_off + a.w + 2;
    float *s_base = reinterpret_cast<float *>(s_lo + a.w + 1);
    __shared__ uint32_t hist[256];
    __shared__ uint64_t okeys[ETF_MAX_TOPK];
    __shared__ uint32_t s_digit, s_rank, s_n, s_total;
    const int64_t q = blockIdx.x;
    if (!a.flag[q]) return;
    if (threadIdx.x == 0) atomicAdd(a.nflag, 1u);
    for (int i = threadIdx.x; i < a.M * a.K; i += 256) tab[i] = a.lut[q * a.M * a.K + i];
    if (threadIdx.x == 0) s_total = 0;
    ivf_setup_lists(a, q, s_off, s_lo, s_base);
    const IvfLists L{s_off, s_lo, s_base, a.w};
    const uint32_t total = s_off[a.w];
    auto dist_of = [&](uint32_t i, uint32_t &e) -> float {
        const int p = L.list_of(i);
        e = s_lo[p] + (i - s_off[p]);
        return ivf_distance(tab, a.ecodes + (int64_t)e * a.M, a.M, a.K, s_base[p] + a.eterm[e]);
    };
    // how many vectors there are at all (capped per entry at k, which is all that can matter)
    {
        uint32_t mine = 0;
        for (uint32_t i = threadIdx.x; i < total; i += 256) {
            const int p = L.list_of(i);
            const uint32_t e = s_lo[p] + (i - s_off[p]);
            mine += min(a.ebegin[e + 1] - a.ebegin[e], (uint32_t)a.k);
        }
        atomicAdd(&s_total, mine);
        __syncthreads();
    }
    const uint32_t k = min((uint32_t)a.k, s_total);  // vectors to return; the rest of the row is padding
    uint64_t prefix = 0;
    uint32_t rank = k;
    if (k > 0) {
        for (int p = 0, shift = 56; p < 8; ++p, shift -= 8) {
            hist[threadIdx.x] = 0;
            __syncthreads();
            for (uint32_t i = threadIdx.x; i < total; i += 256) {
                uint32_t e;
                const uint32_t v = __float_as_uint(dist_of(i, e));
                const uint32_t first = a.ebegin[e];
                const uint32_t mult = min(a.ebegin[e + 1] - first, (uint32_t)a.k);
                if (p < 4) {
                    const int sh = shift - 32;
                    if (p == 0 || (v >> (sh + 8)) == ((uint32_t)(prefix >> 32) >> (sh + 8))) atomicAdd(&hist[(v >> sh) & 255], mult);
                } else if (v == (uint32_t)(prefix >> 32)) {
                    for (uint32_t j = 0; j < mult; ++j) {
                        const uint32_t id = (uint32_t)a.ids[first + j];
                        if (p == 4 || (id >> (shift + 8)) == ((uint32_t)prefix >> (shift + 8))) atomicAdd(&hist[(id >> shift) & 255], 1u);
                    }
                }
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                uint32_t below = 0;
                int b = 0;
                for (; b < 255; ++b) {
                    if (below + hist[b] >= rank) break;
                    below += hist[b];
                }
                s_digit = (uint32_t)b;
                s_rank = rank - below;
            }
            __syncthreads();
            prefix |= (uint64_t)s_digit << shift;
            rank = s_rank;
            __syncthreads();
        }
    }
    if (threadIdx.x == 0) s_n = 0;
    __syncthreads();
    if (k > 0) {
        const uint32_t vk = (uint32_t)(prefix >> 32), idk = (uint32_t)prefix;
        for (uint32_t i = threadIdx.x; i < total; i += 256) {
            uint32_t e;
            const uint32_t v = __float_as_uint(dist_of(i, e));
            if (v > vk) continue;
            const uint32_t first = a.ebegin[e];
            const uint32_t mult = min(a.ebegin[e + 1] - first, (uint32_t)a.k);
            for (uint32_t j = 0; j < mult; ++j) {
                const uint32_t id = (uint32_t)a.ids[first + j];
                if (v < vk || id <= idk) {
                    const uint32_t pos = atomicAdd(&s_n, 1u);
                    if (pos < ETF_MAX_TOPK) okeys[pos] = ((uint64_t)v << 32) | id;
                }
            }
        }
    }
    __syncthreads();
    const int n = (int)min(s_n, (uint32_t)ETF_MAX_TOPK);
    const int n2 = pow2_at_least(max(n, 1));
    for (int i = n + threadIdx.x; i < n2; i += 256) okeys[i] = ~0ull;
    __syncthreads();
    bitonic_sort_u64(okeys, n2);
    for (int i = threadIdx.x; i < a.k; i += 256) {
        const bool have = i < n;
        a.out_ids[q * a.k + i] = have ? (int32_t)(uint32_t)okeys[i] : -1;
        a.out_dist[q * a.k + i] = have ? __uint_as_float((uint32_t)(okeys[i] >> 32)) : __uint_as_float(0x7F800000u);
    }
}

}  // namespace etf

// =============================================================================================
// host side: index build, upload, entry points
// =============================================================================================
namespace {

int64_t ivf_al(int64_t x) { return (x + 255) & ~(int64_t)255; }

void ivf_layout(etf_ctx *ctx)
{
    IvfIndex &iv = ctx->ivf;
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        const int64_t o = off;
        off = ivf_al(off + bytes);
        return o;
    };
    iv.o_centroids = take((int64_t)iv.Kc * ctx->d * 4);
    iv.o_codebooks = take((int64_t)ctx->codebooks.size() * 4);
    iv.o_lbegin = take(((int64_t)iv.Kc + 1) * 4);
    iv.o_ecodes = take(iv.Ne * ctx->M);
    iv.o_eterm = take(iv.Ne * 4);
    iv.o_ebegin = take((iv.Ne + 1) * 4);
    iv.o_ids = take(iv.N * 4);
    iv.total = off;
}

struct IvfPlan {
    int64_t nqb = 0;  // queries per batch
    uint32_t C = 0;
    int64_t o_counter = 0, o_coarse = 0, o_probes = 0, o_lut = 0, o_cnt = 0, o_flag = 0, o_cand = 0, total = 0;
};

int ivf_plan(const etf_ctx *ctx, int64_t Q, int k, int w, IvfPlan &P)
{
    const IvfIndex &iv = ctx->ivf;
    if (!iv.built) return fail(ctx, ETF_ESTATE, "no IVF index: call etf_ivf_build first");
    if (Q <= 0) return fail(ctx, ETF_EINVAL, "Q must be positive");
    if (k < 1 || k > ETF_MAX_TOPK) return fail(ctx, ETF_EINVAL, "need 1 <= k <= %d (k=%d)", ETF_MAX_TOPK, k);
    if (w < 1 || w > iv.Kc || w > 4096) return fail(ctx, ETF_EINVAL, "need 1 <= w <= min(cells, 4096) (w=%d, cells=%d)", w, iv.Kc);
    int64_t C = ctx->opt.cand_cap;
    if (C == 0) {  // the bound's bin is 3 % wide: a few k entries lie below its upper edge
        C = 4096;
        while (C < 8 * (int64_t)k) C <<= 1;
    }
    P.C = (uint32_t)C;
    const int64_t per_q = (int64_t)iv.Kc * 4 + (int64_t)w * 4 + (int64_t)ctx->M * ctx->K * 4 + 8 + C * 8;
    P.nqb = std::max<int64_t>(1, std::min<int64_t>(Q, ctx->opt.ws_cap_bytes / per_q));
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        const int64_t o = off;
        off = ivf_al(off + bytes);
        return o;
    };
    P.o_counter = take(256);
    P.o_coarse = take(P.nqb * iv.Kc * 4);
    P.o_probes = take(P.nqb * w * 4);
    P.o_lut = take(P.nqb * ctx->M * ctx->K * 4);
    P.o_cnt = take(P.nqb * 4);
    P.o_flag = take(P.nqb * 4);
    P.o_cand = take(P.nqb * C * 8);
    P.total = off;
    return ETF_OK;
}

}  // namespace

extern "C" int etf_ivf_set_coarse(etf_ctx *ctx, const float *centroids, int Kc)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->codebooks.empty()) return fail(ctx, ETF_ESTATE, "no codebooks: the residual quantiser gives d");
    if (!centroids || Kc < 1 || Kc > 65536) return fail(ctx, ETF_EINVAL, "need centroids and 1 <= cells <= 65536 (cells=%d)", Kc);
    try {
        ctx->ivf = IvfIndex();
        ctx->ivf.Kc = Kc;
        ctx->ivf.centroids.assign(centroids, centroids + (size_t)Kc * ctx->d);
    } catch (const std::bad_alloc &) {
        return fail(ctx, ETF_ENOMEM, "out of host memory");
    }
    return ETF_OK;
}

extern "C" int etf_ivf_build(etf_ctx *ctx, const int32_t *cells, const uint8_t *codes, int64_t N, const int32_t *ids)
{
    if (!ctx) return ETF_EINVAL;
    IvfIndex &iv = ctx->ivf;
    if (ctx->codebooks.empty() || iv.Kc == 0) return fail(ctx, ETF_ESTATE, "need codebooks and etf_ivf_set_coarse first");
    if (!cells || !codes || N <= 0 || N >= ((int64_t)1 << 31)) return fail(ctx, ETF_EINVAL, "cells or codes is null, or N out of range");
    const int M = ctx->M, K = ctx->K, d = ctx->d, ds = ctx->ds, Kc = iv.Kc;
    for (int64_t i = 0; i < N; ++i) {
        if (cells[i] < 0 || cells[i] >= Kc) return fail(ctx, ETF_EINVAL, "cell %d of vector %lld is outside [0, %d)", cells[i], (long long)i, Kc);
        if (ids && ids[i] < 0) return fail(ctx, ETF_EINVAL, "ids must be non-negative");
        for (int m = 0; m < M; ++m)
            if (codes[i * M + m] >= K) return fail(ctx, ETF_EINVAL, "a code byte is >= K=%d", K);
    }
    try {
        // order by (cell, encoding, id)
        std::vector<int64_t> ord((size_t)N);
        for (int64_t i = 0; i < N; ++i) ord[i] = i;
        auto idof = [&](int64_t i) { return ids ? ids[i] : (int32_t)i; };
        std::sort(ord.begin(), ord.end(), [&](int64_t a, int64_t b) {
            if (cells[a] != cells[b]) return cells[a] < cells[b];
            const int c = memcmp(codes + a * M, codes + b * M, (size_t)M);
            if (c != 0) return c < 0;
            return idof(a) < idof(b);
        });
        iv.built = false;
        iv.N = N;
        iv.lbegin.assign((size_t)Kc + 1, 0);
        iv.ecodes.clear();
        iv.ebegin.clear();
        iv.ids_sorted.resize((size_t)N);
        std::vector<int32_t> ecell;
        for (int64_t r = 0; r < N; ++r) {
            const int64_t i = ord[r];
            iv.ids_sorted[r] = idof(i);
            const bool fresh = r == 0 || cells[i] != cells[ord[r - 1]] || memcmp(codes + i * M, codes + ord[r - 1] * M, (size_t)M) != 0;
            if (fresh) {
                iv.ebegin.push_back((uint32_t)r);
                iv.ecodes.insert(iv.ecodes.end(), codes + i * M, codes + (i + 1) * M);
                ecell.push_back(cells[i]);
                iv.lbegin[cells[i] + 1]++;
            }
        }
        iv.Ne = (int64_t)ecell.size();
        iv.ebegin.push_back((uint32_t)N);
        for (int c = 0; c < Kc; ++c) iv.lbegin[c + 1] += iv.lbegin[c];
        iv.max_list = 0;
        for (int c = 0; c < Kc; ++c) iv.max_list = std::max<int64_t>(iv.max_list, iv.lbegin[c + 1] - iv.lbegin[c]);
        iv.max_dup = 0;
        for (int64_t e = 0; e < iv.Ne; ++e) iv.max_dup = std::max<int64_t>(iv.max_dup, iv.ebegin[e + 1] - iv.ebegin[e]);
        // the entry's constant term ||r||^2 + 2 <c, r> in double, r the reconstructed residual
        iv.eterm.resize((size_t)iv.Ne);
        const float *cb = ctx->codebooks.data();
        parallel_slices(iv.Ne, host_threads(), [&](int, int64_t lo, int64_t hi) {
            for (int64_t e = lo; e < hi; ++e) {
                const float *cen = iv.centroids.data() + (size_t)ecell[e] * d;
                double t = 0.0;
                for (int m = 0; m < M; ++m) {
                    const float *cw = cb + ((size_t)m * K + iv.ecodes[e * M + m]) * ds;
                    for (int j = 0; j < ds; ++j) t += (double)cw[j] * (double)cw[j] + 2.0 * (double)cen[m * ds + j] * (double)cw[j];
                }
                iv.eterm[e] = (float)t;
            }
        });
        // table lookups of one traversal of every list's Encoding Tree (paper: "Statistics of Encoding Tree"): the
        // leaf of an entry sits at level 1 + max(common prefix with its neighbours inside the list) and carries the
        // rest as postfix; the internal nodes are the prefixes shared by at least two entries
        auto lcp = [&](int64_t a, int64_t b) {
            int p = 0;
            while (p < M && iv.ecodes[a * M + p] == iv.ecodes[b * M + p]) ++p;
            return p;
        };
        int64_t lookups = 0;
        for (int c = 0; c < Kc; ++c) {
            const int64_t lo = iv.lbegin[c], hi = iv.lbegin[c + 1];
            int prev = 0;
            for (int64_t e = lo; e < hi; ++e) {
                const int next = e + 1 < hi ? lcp(e, e + 1) : 0;
                const int level = std::min(M, 1 + std::max(prev, next));
                lookups += 1 + (M - level);                                              // the leaf and its postfix
                lookups += std::max(0, std::min(next, M - 1) - std::min(prev, M - 1));   // internal nodes that start here
                prev = next;
            }
        }
        iv.tree_lookups = lookups;
        ivf_layout(ctx);
        iv.dev_base = nullptr;
        iv.built = true;
    } catch (const std::bad_alloc &) {
        ctx->ivf.built = false;
        return fail(ctx, ETF_ENOMEM, "out of host memory");
    }
    return ETF_OK;
}

extern "C" int etf_ivf_stats(const etf_ctx *ctx, etf_ivf_stats_t *out)
{
    if (!ctx) return ETF_EINVAL;
    if (!out) return fail(ctx, ETF_EINVAL, "output pointer is null");
    const IvfIndex &iv = ctx->ivf;
    if (!iv.built) return fail(ctx, ETF_ESTATE, "no IVF index: call etf_ivf_build first");
    out->cells = iv.Kc;
    out->N = iv.N;
    out->entries = iv.Ne;
    out->max_list = iv.max_list;
    out->max_dup = iv.max_dup;
    out->tree_lookups = iv.tree_lookups;
    out->flat_lookups = iv.N * ctx->M;
    out->device_bytes = iv.total;
    return ETF_OK;
}

extern "C" int64_t etf_ivf_device_bytes(const etf_ctx *ctx)
{
    if (!ctx) return ETF_EINVAL;
    if (!ctx->ivf.built) return fail(ctx, ETF_ESTATE, "no IVF index: call etf_ivf_build first");
    return ctx->ivf.total;
}

extern "C" int etf_ivf_upload(etf_ctx *ctx, void *dev_buf, int64_t bytes)
{
    int rc = need_device(ctx);
    if (rc) return rc;
    IvfIndex &iv = ctx->ivf;
    if (!iv.built) return fail(ctx, ETF_ESTATE, "no IVF index: call etf_ivf_build first");
    if (!dev_buf || ((uintptr_t)dev_buf & 255) != 0) return fail(ctx, ETF_EINVAL, "device buffer is null or not 256-byte aligned");
    if (bytes < iv.total) return fail(ctx, ETF_ENOMEM, "device buffer too small: %lld < %lld", (long long)bytes, (long long)iv.total);
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t st = (hipStream_t)ctx->stream;
    char *base = (char *)dev_buf;
    HIP_TRY(ctx, hipMemcpyAsync(base + iv.o_centroids, iv.centroids.data(), iv.centroids.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipMemcpyAsync(base + iv.o_codebooks, ctx->codebooks.data(), ctx->codebooks.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipMemcpyAsync(base + iv.o_lbegin, iv.lbegin.data(), iv.lbegin.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipMemcpyAsync(base + iv.o_ecodes, iv.ecodes.data(), iv.ecodes.size(), hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipMemcpyAsync(base + iv.o_eterm, iv.eterm.data(), iv.eterm.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipMemcpyAsync(base + iv.o_ebegin, iv.ebegin.data(), iv.ebegin.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipMemcpyAsync(base + iv.o_ids, iv.ids_sorted.data(), iv.ids_sorted.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    iv.dev_base = base;
    return ETF_OK;
}

// ---- database side on the device: cell, residual, residual encoding ------------------------------------------
extern "C" int64_t etf_ivf_assign_workspace_bytes(const etf_ctx *ctx, int64_t n)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->codebooks.empty() || ctx->ivf.Kc == 0) return fail(ctx, ETF_ESTATE, "need codebooks and etf_ivf_set_coarse first");
    if (n < 0) return fail(ctx, ETF_EINVAL, "n is negative");
    return ivf_al((int64_t)ctx->ivf.Kc * ctx->d * 4) + ivf_al(etf_encode_workspace_bytes(ctx)) + ivf_al(n * ctx->d * 4);
}

extern "C" int etf_ivf_assign_device(etf_ctx *ctx, const float *x, int64_t n, int32_t *cells_out, uint8_t *codes_out, void *ws,
                                     int64_t ws_bytes)
{
    int rc = need_device(ctx);
    if (rc) return rc;
    if (ctx->codebooks.empty() || ctx->ivf.Kc == 0) return fail(ctx, ETF_ESTATE, "need codebooks and etf_ivf_set_coarse first");
    if (n < 0 || (n > 0 && (!x || !cells_out || !codes_out))) return fail(ctx, ETF_EINVAL, "null input or output with n=%lld", (long long)n);
    if (!ws || ((uintptr_t)ws & 255) != 0) return fail(ctx, ETF_EINVAL, "workspace is null or not 256-byte aligned");
    const int64_t need = etf_ivf_assign_workspace_bytes(ctx, n);
    if (ws_bytes < need) return fail(ctx, ETF_ENOMEM, "workspace too small: %lld < %lld", (long long)ws_bytes, (long long)need);
    if (n == 0) return ETF_OK;
    if (n * ctx->d >= ((int64_t)1 << 38)) return fail(ctx, ETF_EINVAL, "n too large for one call");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t st = (hipStream_t)ctx->stream;
    const IvfIndex &iv = ctx->ivf;
    char *w = (char *)ws;
    float *cent = (float *)w;
    char *enc_ws = w + ivf_al((int64_t)iv.Kc * ctx->d * 4);
    const int64_t enc_bytes = ivf_al(etf_encode_workspace_bytes(ctx));
    float *res = (float *)(enc_ws + enc_bytes);
    HIP_TRY(ctx, hipMemcpyAsync(cent, iv.centroids.data(), iv.centroids.size() * 4, hipMemcpyHostToDevice, st));
    {
        ProfScope prof(ctx, ETF_K_ENCODE);
        hipLaunchKernelGGL(k_ivf_coarse<true>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x, n, ctx->d, cent, iv.Kc, nullptr, cells_out, iv.Kc);
        LAUNCH_CHECK(ctx, "k_ivf_coarse");
        hipLaunchKernelGGL(k_ivf_residual, dim3((unsigned)((n * ctx->d + 255) / 256)), dim3(256), 0, st, x, n, ctx->d, cent, cells_out, res);
        LAUNCH_CHECK(ctx, "k_ivf_residual");
    }
    return etf_pq_encode_device(ctx, res, n, codes_out, enc_ws, enc_bytes);
}

// ---- search ---------------------------------------------------------------------------------------------
extern "C" int64_t etf_ivf_workspace_bytes(const etf_ctx *ctx, int64_t Q, int k, int w)
{
    if (!ctx) return ETF_EINVAL;
    IvfPlan P;
    int rc = ivf_plan(ctx, Q, k, w, P);
    if (rc) return rc;
    return P.total;
}

extern "C" int etf_ivf_search(etf_ctx *ctx, const float *queries, int64_t Q, int k, int w, int32_t *out_ids, float *out_dist,
                              void *ws, int64_t ws_bytes)
{
    int rc = need_device(ctx);
    if (rc) return rc;
    IvfIndex &iv = ctx->ivf;
    if (!iv.built) return fail(ctx, ETF_ESTATE, "no IVF index: call etf_ivf_build first");
    if (!iv.dev_base) return fail(ctx, ETF_ESTATE, "IVF index not on the device: call etf_ivf_upload first");
    if (!queries || !out_ids || !out_dist) return fail(ctx, ETF_EINVAL, "null pointer");
    if (!ws || ((uintptr_t)ws & 255) != 0) return fail(ctx, ETF_EINVAL, "workspace is null or not 256-byte aligned");
    IvfPlan P;
    rc = ivf_plan(ctx, Q, k, w, P);
    if (rc) return rc;
    if (ws_bytes < P.total) return fail(ctx, ETF_ENOMEM, "workspace too small: %lld < %lld", (long long)ws_bytes, (long long)P.total);
    const int M = ctx->M, K = ctx->K, d = ctx->d;
    const size_t lds_scan = ivf_lds_bytes(M, K, w, true), lds_exact = ivf_lds_bytes(M, K, w, false);
    if (lds_scan > 150 * 1024) return fail(ctx, ETF_EINVAL, "w=%d with M=%d K=%d needs %zu bytes of LDS", w, M, K, lds_scan);
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t st = (hipStream_t)ctx->stream;
    char *wsp = (char *)ws;
    const char *img = iv.dev_base;
    uint32_t *counter = reinterpret_cast<uint32_t *>(wsp + P.o_counter);
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, counter, (int64_t)64, 0u);
    LAUNCH_CHECK(ctx, "k_fill_u32");
    ctx->last_flag_count = counter;
    rc = set_lds(ctx, k_ivf_scan, lds_scan);
    if (rc) return rc;
    rc = set_lds(ctx, k_ivf_exact, lds_exact);
    if (rc) return rc;
    const float *cent = reinterpret_cast<const float *>(img + iv.o_centroids);
    const float *cbd = reinterpret_cast<const float *>(img + iv.o_codebooks);
    ChunkOrder ord;
    for (int j = 0; j < ETF_MAX_M; ++j) ord.src[j] = (uint8_t)j;
    for (int64_t q0 = 0; q0 < Q; q0 += P.nqb) {
        const int64_t nq = std::min<int64_t>(P.nqb, Q - q0);
        const float *qb = queries + q0 * d;
        float *coarse = reinterpret_cast<float *>(wsp + P.o_coarse);
        int32_t *probes = reinterpret_cast<int32_t *>(wsp + P.o_probes);
        float *lut = reinterpret_cast<float *>(wsp + P.o_lut);
        uint32_t *cnt = reinterpret_cast<uint32_t *>(wsp + P.o_cnt);
        uint32_t *flag = reinterpret_cast<uint32_t *>(wsp + P.o_flag);
        uint64_t *cand = reinterpret_cast<uint64_t *>(wsp + P.o_cand);
        {
            ProfScope prof(ctx, ETF_K_IVF_COARSE);
            // about 2048 workgroups: the centroids in slices of whole tiles of 32
            const int64_t qblocks = (nq + 255) / 256;
            int64_t slices = std::max<int64_t>(1, std::min<int64_t>((iv.Kc + 31) / 32, 2048 / qblocks));
            const int cslice = (int)(((iv.Kc + slices - 1) / slices + 31) / 32 * 32);
            slices = (iv.Kc + cslice - 1) / cslice;
            hipLaunchKernelGGL(k_ivf_coarse<false>, dim3((unsigned)qblocks, (unsigned)slices), dim3(256), 0, st, qb, nq, d, cent, iv.Kc, coarse,
                               nullptr, cslice);
            LAUNCH_CHECK(ctx, "k_ivf_coarse");
            hipLaunchKernelGGL(k_ivf_probe, dim3((unsigned)nq), dim3(256), (size_t)pow2_at_least_host(w) * 8, st, coarse, iv.Kc, w, probes);
            LAUNCH_CHECK(ctx, "k_ivf_probe");
        }
        {
            // tables of scalar products <q_m, codeword>, one set per query, shared by all cells
            ProfScope prof(ctx, ETF_K_LUT);
            const int64_t tiles = (nq + QT - 1) / QT;
            hipLaunchKernelGGL(k_lut_mfma<true>, dim3((unsigned)tiles, (unsigned)M), dim3(256), 0, st, qb, nq, (int64_t)0, d, M, K, cbd, nullptr,
                               nullptr, nullptr, ctx->dsp, nullptr, lut, ord);
            LAUNCH_CHECK(ctx, "k_lut_mfma");
        }
        const unsigned fb = (unsigned)((nq + 255) / 256);
        hipLaunchKernelGGL(k_fill_u32, dim3(fb), dim3(256), 0, st, flag, nq, ctx->opt.force_fallback ? 1u : 0u);
        hipLaunchKernelGGL(k_fill_u32, dim3(fb), dim3(256), 0, st, cnt, nq, 0u);
        LAUNCH_CHECK(ctx, "k_fill_u32");
        IvfScanArgs a;
        memset(&a, 0, sizeof a);
        a.lut = lut;
        a.coarse = coarse;
        a.probes = probes;
        a.M = M;
        a.K = K;
        a.Kc = iv.Kc;
        a.w = w;
        a.k = k;
        a.lbegin = reinterpret_cast<const uint32_t *>(img + iv.o_lbegin);
        a.ecodes = reinterpret_cast<const uint8_t *>(img + iv.o_ecodes);
        a.eterm = reinterpret_cast<const float *>(img + iv.o_eterm);
        a.ebegin = reinterpret_cast<const uint32_t *>(img + iv.o_ebegin);
        a.ids = reinterpret_cast<const int32_t *>(img + iv.o_ids);
        a.cnt = cnt;
        a.cand = cand;
        a.C = P.C;
        a.flag = flag;
        a.nflag = counter;
        a.out_ids = out_ids + q0 * k;
        a.out_dist = out_dist + q0 * k;
        if (!ctx->opt.force_fallback) {
            ProfScope prof(ctx, ETF_K_IVF_SCAN);
            hipLaunchKernelGGL(k_ivf_scan, dim3((unsigned)nq), dim3(256), lds_scan, st, a);
            LAUNCH_CHECK(ctx, "k_ivf_scan");
        }
        SelectArgs sa;
        memset(&sa, 0, sizeof sa);
        sa.cnt = cnt;
        sa.cand = cand;
        sa.C = P.C;
        sa.ebegin = a.ebegin;
        sa.ids = a.ids;
        sa.k = k;
        sa.out_ids = a.out_ids;
        sa.out_dist = a.out_dist;
        sa.flag = flag;
        sa.allow_short = 1;
        {
            ProfScope prof(ctx, ETF_K_SELECT);
            hipLaunchKernelGGL(k_select, dim3((unsigned)nq), dim3(256), select_lds_bytes(k), st, sa);
            LAUNCH_CHECK(ctx, "k_select");
        }
        {
            ProfScope prof(ctx, ETF_K_EXACT);
            hipLaunchKernelGGL(k_ivf_exact, dim3((unsigned)nq), dim3(256), lds_exact, st, a);
            LAUNCH_CHECK(ctx, "k_ivf_exact");
        }
    }
    return ETF_OK;
}
