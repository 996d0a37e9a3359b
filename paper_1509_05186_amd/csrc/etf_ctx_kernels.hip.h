// Tree traversal with the distance context in registers (gfx950, wave64).  Included only by etf_device.hip.
//
// The paper walks the tree depth first and keeps a "Distance Context": the partial sum of every level
// on the current path, so that a node costs one lookup and one add (section "Distance Computation with
// Hierarchical Memory Structure").  Depth-first order of the leaves is the lexicographic order of the
// encodings, and the depth at which a leaf's path leaves the previous leaf's path is their longest
// common prefix.  So a wave that walks a run of the sorted (sub-)encodings with the context of its 64
// queries in VGPRs (lane = query) does exactly the tree's work: for a leaf whose common prefix with its
// predecessor is p chunks it does D - p lookups, which over all leaves is the number of nodes plus
// postfix chunks of the encoding tree; only the first leaf of every run pays for the whole path.
// Compared with the level-synchronous kernels, no partial sum of an internal node ever goes to memory.
//
// Everything inside a batch of leaves is branch free: a level that is not recomputed loads row 0 of
// the table slice (resident in L1) and keeps its old value by mask arithmetic, so that all the loads
// of a batch are issued back to back.
#pragma once

#include "etf_kernels.hip.h"

namespace etf {

// all-ones if a >= b else 0, for small non-negative ints, without a compare (stays on the scalar unit)
__device__ __forceinline__ uint32_t mask_ge(int a, int b) { return (uint32_t)((b - a - 1) >> 31); }

// number of leading chunks (bytes, lowest byte first) in which two padded code records agree
template <int NDW>
__device__ __forceinline__ int common_prefix(const uint32_t a[NDW], const uint32_t b[NDW])
{
    int p = 4 * NDW;
#pragma unroll
    for (int i = NDW - 1; i >= 0; --i) {
        const uint32_t x = a[i] ^ b[i];
        p = x ? 4 * i + ((__ffs((int)x) - 1) >> 3) : p;
    }
    return p;
}

// One batch of UB consecutive items of a 64-item chunk.  Lane i of the chunk holds the padded code record
// my_dw and the common prefix my_lcp of item i; the wave walks items s0 .. s0+UB-1.
//   ctx[l]   partial sum down to level l+1 of the path of the previous item (per lane = per query)
//   lut      this tile's table slice of the tree's first chunk, already offset by the lane
//   res[u]   receives the full-depth sum of item s0+u
template <int DT, int NDW>
__device__ __forceinline__ void ctx_batch(float ctx[DT], const float *__restrict__ lut, int K, int D,
                                          const uint32_t my_dw[NDW], int my_lcp, int s0, int cnt, float res[UB])
{
    float x[UB][DT];
    int lcp[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) {
        const int src = min(s0 + u, cnt - 1);
        // beyond the end of the chunk: nothing is recomputed (prefix = D)
        const uint32_t live = mask_ge(cnt - 1, s0 + u);
        lcp[u] = (int)(((uint32_t)__builtin_amdgcn_readlane(my_lcp, src) & live) | ((uint32_t)D & ~live));
        uint32_t dw[NDW];
#pragma unroll
        for (int i = 0; i < NDW; ++i) dw[i] = (uint32_t)__builtin_amdgcn_readlane((int)my_dw[i], src);
#pragma unroll
        for (int l = 0; l < DT; ++l) {
            const uint32_t code = (dw[l >> 2] >> (8 * (l & 3))) & 255u;
            const uint32_t act = mask_ge(l, lcp[u]) & mask_ge(D - 1, l);  // level is real and below the common prefix
            x[u][l] = lut[(int64_t)(((uint32_t)l * (uint32_t)K + code) & act) * QT];
        }
    }
#pragma unroll
    for (int u = 0; u < UB; ++u) {
#pragma unroll
        for (int l = 0; l < DT; ++l) {
            const uint32_t real = mask_ge(D - 1, l);
            const uint32_t upd = mask_ge(l, lcp[u]) | ~real;  // levels past D just copy the level above
            const float add = __uint_as_float(__float_as_uint(x[u][l]) & real);
            const float above = l == 0 ? 0.f : ctx[l - 1];
            ctx[l] = run_pick(above + add, ctx[l], upd);
        }
        res[u] = ctx[DT - 1];
    }
}

// ------------------------------------------------------------------------------------------------
// S2+S3 of one tree in one pass: leafp[i] = sum over the tree's D chunks of LUT(chunk value of the i-th
//     distinct sub-encoding), the partial sums of shared prefixes carried in registers.
//     codes [U][4*NDW] padded records in lexicographic order; out [tile][U][64].
//     grid (blocks, tiles), block 256; every wave takes `per_wave` (a multiple of 64) consecutive leaves.
// ------------------------------------------------------------------------------------------------
template <int DT, int NDW>
__global__ __launch_bounds__(256) void k_tree_ctx(const uint32_t *__restrict__ codes, int64_t U, float *__restrict__ out,
                                                  const float *__restrict__ lutT, int M, int K, int m0, int D,
                                                  int per_wave)
{
    const int tile = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int64_t wv = (int64_t)blockIdx.x * 4 + uniform(threadIdx.x >> 6);
    const int64_t lo = wv * per_wave;
    const int64_t hi = min(U, lo + per_wave);
    const float *lut = lutT + ((int64_t)tile * M + m0) * K * QT + lane;
    float *orow = out + (int64_t)tile * U * QT + lane;
    float ctx[DT];
#pragma unroll
    for (int l = 0; l < DT; ++l) ctx[l] = 0.f;
    for (int64_t base = lo; base < hi; base += 64) {
        const int cnt = (int)min<int64_t>(64, hi - base);
        uint32_t my_dw[NDW], before[NDW];
#pragma unroll
        for (int i = 0; i < NDW; ++i) my_dw[i] = lane < cnt ? codes[(base + lane) * NDW + i] : 0u;
        // predecessor's record: previous lane, or (lane 0) the last leaf of the previous chunk
#pragma unroll
        for (int i = 0; i < NDW; ++i) {
            const uint32_t up = (uint32_t)__shfl_up((int)my_dw[i], 1);
            before[i] = (lane == 0 && base > lo) ? codes[(base - 1) * NDW + i] : up;
        }
        int my_lcp = min(common_prefix<NDW>(my_dw, before), D);
        if (lane == 0 && base == lo) my_lcp = 0;  // first leaf of the run: whole path
        for (int s0 = 0; s0 < cnt; s0 += UB) {
            float res[UB];
            ctx_batch<DT, NDW>(ctx, lut, K, D, my_dw, my_lcp, s0, cnt, res);
#pragma unroll
            for (int u = 0; u < UB; ++u)
                if (s0 + u < cnt) orow[(base + s0 + u) * QT] = res[u];
        }
    }
}

// ------------------------------------------------------------------------------------------------
// S3(tree 0) + S4 fused: distance of every distinct encoding = tree 0's sum, carried in registers as
//     above over the first D0 chunks of the sorted full encodings, plus the rows of the other trees'
//     result tables (paper "Encoding Forests": per-tree results summed per vector, in tree order).
//     With a single tree there is nothing to gather and this kernel is the whole traversal.
//     items: FILTER -> distinct encodings in order; SAMPLE -> sample_enc[i]; ALLPAIRS -> enc_of_pos[n].
//     The last two visit encodings in arbitrary order, so every item recomputes its whole path.
//     r.leafp[t], r.leaf_of[t], r.U[t] for t = 1 .. T-1 are the other trees (slot 0 is unused; slots
//     t >= T are valid padding); codes0 [Nd][4*NDW] are the padded tree-0 records.
//     grid (blocks, tiles), block 256.
// ------------------------------------------------------------------------------------------------
template <int MODE, int DT, int NDW, int TMAX>
__global__ __launch_bounds__(256) void k_fused(const uint32_t *__restrict__ codes0, int D0, const float *__restrict__ lutT,
                                               int M, int K, ReduceArgs r, int64_t nitems,
                                               const uint32_t *__restrict__ map, int per_wave, OutArgs o)
{
    const int tile = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int w = uniform(threadIdx.x >> 6);
    const int64_t wv = (int64_t)blockIdx.x * 4 + w;
    const int64_t lo = wv * per_wave;
    const int64_t hi = min(nitems, lo + per_wave);
    const float *lut = lutT + (int64_t)tile * M * K * QT + lane;
    __shared__ float tbuf[MODE == OUT_ALLPAIRS ? 4 : 1][MODE == OUT_ALLPAIRS ? 64 : 1][65];
    constexpr int STG = 8;
    __shared__ uint64_t stage[MODE == OUT_FILTER ? 4 : 1][MODE == OUT_FILTER ? STG : 1][64];
    int nloc = 0;
    const int64_t ql = (int64_t)tile * QT + lane;
    auto flush = [&]() {
        const uint32_t pos = atomicAdd(&o.cnt[ql], (uint32_t)nloc);
        for (int i = 0; i < nloc; ++i)
            if (pos + i < o.C) o.cand[ql * o.C + pos + i] = stage[w][i][lane];
        nloc = 0;
    };
    float tauv = 0.f, best = __uint_as_float(0x7F800000u);
    if (MODE == OUT_FILTER) tauv = o.tau[ql];
    float ctx[DT];
#pragma unroll
    for (int l = 0; l < DT; ++l) ctx[l] = 0.f;
    for (int64_t base = lo; base < hi; base += 64) {
        const int cnt = (int)min<int64_t>(64, hi - base);
        const bool live = lane < cnt;
        const uint32_t e = live ? (MODE == OUT_FILTER ? (uint32_t)(base + lane) : map[base + lane]) : 0u;
        uint32_t my_dw[NDW];
#pragma unroll
        for (int i = 0; i < NDW; ++i) my_dw[i] = live ? codes0[(int64_t)e * NDW + i] : 0u;
        int my_lcp = 0;
        if (MODE == OUT_FILTER) {
            uint32_t before[NDW];
#pragma unroll
            for (int i = 0; i < NDW; ++i) {
                const uint32_t up = (uint32_t)__shfl_up((int)my_dw[i], 1);
                before[i] = (lane == 0 && base > lo) ? codes0[(base - 1) * NDW + i] : up;
            }
            my_lcp = min(common_prefix<NDW>(my_dw, before), D0);
            if (lane == 0 && base == lo) my_lcp = 0;
        }
        uint32_t my_rows[TMAX];
#pragma unroll
        for (int t = 1; t < TMAX; ++t) my_rows[t] = live ? r.leaf_of[t][e] : 0u;
        for (int s0 = 0; s0 < cnt; s0 += UB) {
            // rows of the other trees first (the long-latency loads), then tree 0's lookups
            float v[UB][TMAX];
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int src = min(s0 + u, cnt - 1);
#pragma unroll
                for (int t = 1; t < TMAX; ++t) {
                    const uint32_t row = (uint32_t)__builtin_amdgcn_readlane((int)my_rows[t], src);
                    v[u][t] = r.leafp[t][((int64_t)tile * r.U[t] + row) * QT + lane];
                }
            }
            float d[UB];
            ctx_batch<DT, NDW>(ctx, lut, K, D0, my_dw, my_lcp, s0, cnt, d);
#pragma unroll
            for (int u = 0; u < UB; ++u) {
#pragma unroll
                for (int t = 1; t < TMAX; ++t) d[u] += (t < r.T) ? v[u][t] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                if (s0 + u >= cnt) break;
                if (MODE == OUT_ALLPAIRS) tbuf[w][s0 + u][lane] = d[u];
                else if (MODE == OUT_SAMPLE) best = fminf(best, d[u]);
                else if (d[u] <= tauv) {
                    stage[w][nloc][lane] = ((uint64_t)__float_as_uint(d[u]) << 32) | (uint32_t)(base + s0 + u);
                    if (++nloc == STG) flush();
                }
            }
        }
        if (MODE == OUT_ALLPAIRS) {
            __builtin_amdgcn_wave_barrier();
            for (int qq = 0; qq < 64; ++qq) {
                const int64_t q = (int64_t)tile * QT + qq;
                if (q < o.nq && lane < cnt) o.dist[q * o.N + base + lane] = tbuf[w][lane][qq];
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    if (MODE == OUT_FILTER && nloc > 0) flush();
    if (MODE == OUT_SAMPLE && lo < hi) o.gmin[((int64_t)tile * o.ngroups + wv) * QT + lane] = best;
}

}  // namespace etf
