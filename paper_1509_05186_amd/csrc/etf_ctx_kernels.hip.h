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
// Instruction budget.  One CU issues about one wave-wide vector instruction and one scalar instruction
// per clock, and at HBM speed it has about 30 clocks per 256-byte row.  So everything that depends on the
// item but not on the query is computed once per 64 items with lane = item (record bytes, common prefix,
// byte offsets of the table rows, masks), and the walk over the items only broadcasts those values
// (v_readlane) into the scalar offset of buffer loads.  Inside a batch of UBT items nothing branches: a
// level that is not recomputed reads row 0 of its slice and keeps its value through a bit-select, so all
// loads of the batch are issued back to back.  Between batches one uniform branch picks how many of the
// deepest levels the batch touches at all (most batches only the last two).
#pragma once

#include "etf_kernels.hip.h"

namespace etf {

// (a & m) | (b & ~m)
__device__ __forceinline__ float bit_select(uint32_t m, float a, float b)
{
    return __uint_as_float((__float_as_uint(a) & m) | (__float_as_uint(b) & ~m));
}

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

// Records are padded at the FRONT to the unrolled depth DT (1, 2, 4, 8 or 16): slot s of a record is level
// s - pad of the tree, pad = DT - D, and slots below pad are zero in every record.  The common prefix of
// two records therefore counts the padding, a slot below pad is never recomputed, its context stays 0, and
// the deepest level is always slot DT-1.  That makes the split below a compile-time one: the table slices
// of the NL deepest levels (where almost all lookups of a tree fall: own chunks and postfixes of the
// leaves) are staged in LDS, the lookups of the levels above read the transposed tables in global memory
// (L2).  NL = 2 (128 KB, next to the candidate ring) except for the all-pairs output, whose transpose
// buffer takes the room: NL = 0 there.

// copies the NL deepest slices of a tree (chunks m0+D-NL .. m0+D-1, adjacent rows of lutT) into LDS
template <int NL>
__device__ __forceinline__ void stage_deepest(float *lds, const float *__restrict__ lutT, int tile, int M, int K, int m0,
                                              int D)
{
    if (NL == 0) return;
    const float4 *src = reinterpret_cast<const float4 *>(lutT + ((int64_t)tile * M + m0 + D - NL) * K * QT);
    float4 *dst = reinterpret_cast<float4 *>(lds);
    const int total = NL * K * QT / 4;
    for (int i = threadIdx.x; i < total; i += blockDim.x) dst[i] = src[i];
    __syncthreads();
}

// Per-item values of a 64-item chunk, held by the lane that owns the item.
template <int DT>
struct ChunkMeta {
    uint32_t off[DT];  // byte offset of the row each slot reads (0 where the slot is not recomputed)
    uint32_t bits;     // bit s set: slot s is recomputed (s >= common prefix with the predecessor)
    uint32_t deep;     // rows of the two deepest slots inside the staged slices: slot DT-2 | slot DT-1 << 16
    int gmin;          // smallest common prefix among the UBT items of this item's batch
};

// codes: the record array the chunk's items come from (to fetch the predecessor of the chunk's first
// item); `sequential` is false when items are visited in arbitrary order (whole path for every item).
template <int DT, int NDW, int NL, int UBT>
__device__ __forceinline__ void chunk_meta(ChunkMeta<DT> &m, const uint32_t my_dw[NDW], const uint32_t *__restrict__ codes,
                                           int64_t base, int64_t lo, int lane, int cnt, int pad, int K, bool sequential)
{
    int lcp = pad;
    if (sequential) {
        uint32_t before[NDW];
#pragma unroll
        for (int i = 0; i < NDW; ++i) {
            const uint32_t up = (uint32_t)__shfl_up((int)my_dw[i], 1);
            before[i] = (lane == 0 && base > lo) ? codes[(base - 1) * NDW + i] : up;
        }
        lcp = max(min(common_prefix<NDW>(my_dw, before), DT), pad);
        if (lane == 0 && base == lo) lcp = pad;  // first item of the wave's run: whole path
    }
    if (lane >= cnt) lcp = DT;
    m.bits = (0xFFFFFFFFu << lcp) & ((1u << DT) - 1u);
#pragma unroll
    for (int s = 0; s < DT; ++s) {
        const uint32_t code = (my_dw[s >> 2] >> (8 * (s & 3))) & 255u;
        const uint32_t row = (s >= DT - NL) ? (uint32_t)(s - (DT - NL)) * (uint32_t)K + code
                                            : (uint32_t)(s - pad) * (uint32_t)K + code;
        m.off[s] = ((m.bits >> s) & 1u) ? row * (uint32_t)(QT * 4) : 0u;
    }
    m.deep = 0u;
    if (DT >= 2 && NL == 2) {
        const uint32_t c2 = (my_dw[(DT - 2) >> 2] >> (8 * ((DT - 2) & 3))) & 255u;
        const uint32_t c3 = (my_dw[(DT - 1) >> 2] >> (8 * ((DT - 1) & 3))) & 255u;
        m.deep = c2 | (((uint32_t)K + c3) << 16);
    }
    int g = lcp;
#pragma unroll
    for (int d = 1; d < UBT; d <<= 1) g = min(g, __shfl_xor(g, d));
    m.gmin = g;
}

// The common case: no item of the batch leaves the path of its predecessor above the two deepest levels.
// Those two are then simply looked up for every item (both slices are in LDS): the same sum as a masked
// update, without any mask, and per item one broadcast, two LDS reads and two adds.  Items past the end
// of the chunk look up rows of code 0 and leave a meaningless context behind, which nobody reads: a short
// chunk is the last one of the wave's run.
template <int DT, int UBT, class Mid>
__device__ __forceinline__ void ctx_batch_deep(float ctx[DT], const char *ldsb, int lane4, const ChunkMeta<DT> &m, int s0,
                                               int cnt, float res[UBT], Mid mid)
{
    float x2[UBT], x3[UBT];
#pragma unroll
    for (int u = 0; u < UBT; ++u) {
        const uint32_t p = (uint32_t)__builtin_amdgcn_readlane((int)m.deep, s0 + u);
        x2[u] = *reinterpret_cast<const float *>(ldsb + ((p & 0xFFFFu) << 8) + lane4);
        x3[u] = *reinterpret_cast<const float *>(ldsb + ((p >> 16) << 8) + lane4);
    }
    mid();
    const float above = DT >= 3 ? ctx[DT >= 3 ? DT - 3 : 0] : 0.f;
#pragma unroll
    for (int u = 0; u < UBT; ++u) {
        ctx[DT - 2] = above + x2[u];
        ctx[DT - 1] = ctx[DT - 2] + x3[u];
        res[u] = ctx[DT - 1];
    }
}

// One batch of UBT consecutive items (s0 is a multiple of UBT), slots F .. DT-1 only: the caller has checked
// that no item of the batch has a common prefix below F.
//   ctx[s]   partial sum down to slot s of the path of the previous item (per lane = per query)
//   lutr     buffer over this tile's table slices starting at the tree's first chunk
//   ldsb     the NL deepest slices in LDS, as bytes
//   res[u]   receives the full-depth sum of item s0+u
// Items past the end of the chunk (only at the end of a wave's run) have no bit set and read row 0.
// `mid` runs between the issue of the batch's lookups and their use (the place to request data for later).
template <int DT, int NL, int UBT, int F, class Mid>
__device__ __forceinline__ void ctx_batch(float ctx[DT], rsrc_t lutr, const char *ldsb, int lane4, const ChunkMeta<DT> &m,
                                          int s0, int cnt, float res[UBT], Mid mid)
{
    float x[UBT][DT];
    uint32_t bits[UBT];
#pragma unroll
    for (int u = 0; u < UBT; ++u) {
        const int src = s0 + u;
        bits[u] = (uint32_t)__builtin_amdgcn_readlane((int)m.bits, src);
#pragma unroll
        for (int s = F; s < DT; ++s) {
            const int so = __builtin_amdgcn_readlane((int)m.off[s], src);
            if (s >= DT - NL)
                x[u][s] = *reinterpret_cast<const float *>(ldsb + so + lane4);
            else
                x[u][s] = buf_load(lutr, lane4, so);
        }
    }
    mid();
#pragma unroll
    for (int u = 0; u < UBT; ++u) {
#pragma unroll
        for (int s = F; s < DT; ++s) {
            const uint32_t upd = (uint32_t)(-(int)((bits[u] >> s) & 1u));
            const float above = s == 0 ? 0.f : ctx[s - 1];
            ctx[s] = bit_select(upd, above + x[u][s], ctx[s]);
        }
        res[u] = ctx[DT - 1];
    }
}

// picks the cheapest evaluation the batch allows: the last two slots, the deeper half, or all DT slots
template <int DT, int NL, int UBT, class Mid>
__device__ __forceinline__ void ctx_batch_any(float ctx[DT], rsrc_t lutr, const char *ldsb, int lane4,
                                              const ChunkMeta<DT> &m, int s0, int cnt, float res[UBT], Mid mid)
{
    const int gmin = __builtin_amdgcn_readlane(m.gmin, s0);
    constexpr int F1 = DT >= 8 ? DT / 2 : 0;
    if (DT >= 2 && NL == 2 && gmin >= DT - 2) ctx_batch_deep<DT, UBT>(ctx, ldsb, lane4, m, s0, cnt, res, mid);
    else if (F1 > 0 && gmin >= F1) ctx_batch<DT, NL, UBT, F1>(ctx, lutr, ldsb, lane4, m, s0, cnt, res, mid);
    else ctx_batch<DT, NL, UBT, 0>(ctx, lutr, ldsb, lane4, m, s0, cnt, res, mid);
}

// ------------------------------------------------------------------------------------------------
// S2+S3 of one tree in one pass: leafp[i] = sum over the tree's D chunks of LUT(chunk value of the i-th
//     distinct sub-encoding), the partial sums of shared prefixes carried in registers.
//     codes [U][4*NDW] front-padded records in lexicographic order; out [tile][U][64], U*256 < 2^32.
//     grid (blocks, tiles), block 1024, dynamic LDS NL*K*256 bytes; every wave takes `per_wave`
//     (a multiple of 64) consecutive leaves.
// ------------------------------------------------------------------------------------------------
template <int DT, int NDW, int NL, int UBT>
__global__ __launch_bounds__(1024) void k_tree_ctx(const uint32_t *__restrict__ codes, int64_t U, float *__restrict__ out,
                                                   const float *__restrict__ lutT, int M, int K, int m0, int D,
                                                   int per_wave)
{
    extern __shared__ float lds[];
    const int tile = blockIdx.y;
    stage_deepest<NL>(lds, lutT, tile, M, K, m0, D);
    const int lane = threadIdx.x & 63, lane4 = lane * 4;
    const int pad = DT - D;
    const int64_t wv = (int64_t)blockIdx.x * (blockDim.x >> 6) + uniform(threadIdx.x >> 6);
    const int64_t lo = wv * per_wave;
    const int64_t hi = min(U, lo + per_wave);
    const rsrc_t lutr = make_rsrc(lutT + ((int64_t)tile * M + m0) * K * QT, (uint32_t)(D * K * QT * 4));
    const rsrc_t outr = make_rsrc(out + (int64_t)tile * U * QT, (uint32_t)(U * QT * 4));
    const char *ldsb = reinterpret_cast<const char *>(lds);
    float ctx[DT];
#pragma unroll
    for (int s = 0; s < DT; ++s) ctx[s] = 0.f;
    for (int64_t base = lo; base < hi; base += 64) {
        const int cnt = uniform((int)min<int64_t>(64, hi - base));
        uint32_t my_dw[NDW];
#pragma unroll
        for (int i = 0; i < NDW; ++i) my_dw[i] = lane < cnt ? codes[(base + lane) * NDW + i] : 0u;
        ChunkMeta<DT> m;
        chunk_meta<DT, NDW, NL, UBT>(m, my_dw, codes, base, lo, lane, cnt, pad, K, true);
        for (int s0 = 0; s0 < cnt; s0 += UBT) {
            float res[UBT];
            ctx_batch_any<DT, NL, UBT>(ctx, lutr, ldsb, lane4, m, s0, cnt, res, [] {});
            const int so = (int)((base + s0) * (QT * 4));
#pragma unroll
            for (int u = 0; u < UBT; ++u)
                if (s0 + u < cnt) buf_store(res[u], outr, lane4 + u * (QT * 4), so);
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
//     t >= T are valid padding; U[t]*256 < 2^32); codes0 [Nd][4*NDW] are the front-padded tree-0 records.
//
//     The rows of the other trees are random 256-byte reads from HBM, a few microseconds each, while a
//     batch of items is evaluated in a fraction of that.  So they are requested GP items ahead (a whole
//     group of the 64-item chunk, across chunk boundaries too) into registers; the table lookups of the
//     items in between come from LDS, whose counter is separate, so waiting for them does not wait for
//     the rows in flight.  Candidates that pass the bound are compacted into a ring of the wave in LDS
//     (rank of a lane among the passing ones from the ballot) and appended to the queries' lists, one
//     atomic each, by all 64 lanes together when the ring is nearly full and at the end: an atomic with
//     a return value in the item loop would drain the rows in flight every time.
//     grid (blocks, tiles); FILTER and SAMPLE: block 1024, NL = 2; ALLPAIRS: block 256, NL = 0;
//     dynamic LDS NL*K*256 bytes.
// ------------------------------------------------------------------------------------------------
template <int MODE, int DT, int NDW, int TMAX, int NL, int UBT>
__global__ __launch_bounds__(1024) void k_fused(const uint32_t *__restrict__ codes0, int D0, const float *__restrict__ lutT,
                                                int M, int K, ReduceArgs r, int64_t nitems,
                                                const uint32_t *__restrict__ map, int per_wave, OutArgs o)
{
    constexpr int NG1 = TMAX - 1;                              // tables gathered per item
#ifndef ETF_GP
#define ETF_GP 16
#endif
    constexpr int GP = NG1 == 1 ? ETF_GP : UBT;                // items per gather group (GP * NG1 rows in flight)
    constexpr int NGRP = 64 / GP, NBAT = GP / UBT;
    constexpr int NV = NG1 > 0 ? NG1 : 1;
    constexpr int RING = 192;                                  // candidates a wave holds back in LDS
    extern __shared__ float lds[];
    const int tile = blockIdx.y;
    stage_deepest<NL>(lds, lutT, tile, M, K, 0, D0);
    const int lane = threadIdx.x & 63, lane4 = lane * 4;
    const int pad = DT - D0;
    const int w = uniform(threadIdx.x >> 6);
    const int64_t wv = (int64_t)blockIdx.x * (blockDim.x >> 6) + w;
    const int64_t lo = wv * per_wave;
    const int64_t hi = min(nitems, lo + per_wave);
    if (lo >= hi) return;
    const rsrc_t lutr = make_rsrc(lutT + (int64_t)tile * M * K * QT, (uint32_t)(D0 * K * QT * 4));
    rsrc_t tabr[TMAX];
#pragma unroll
    for (int t = 1; t < TMAX; ++t) tabr[t] = make_rsrc(r.leafp[t] + (int64_t)tile * r.U[t] * QT, (uint32_t)(r.U[t] * QT * 4));
    const char *ldsb = reinterpret_cast<const char *>(lds);
    // all-pairs output is transposed through LDS, 4 waves per block in that mode
    __shared__ float tbuf[MODE == OUT_ALLPAIRS ? 4 : 1][MODE == OUT_ALLPAIRS ? 64 : 1][65];
    const int64_t ql = (int64_t)tile * QT + lane;
    // candidates of this wave waiting to be appended: (distance bits << 32) | lane << 26 | item
    __shared__ uint64_t ring[MODE == OUT_FILTER ? 16 : 1][MODE == OUT_FILTER ? RING : 1];
    __shared__ uint32_t wpos[MODE == OUT_FILTER ? 16 : 1][64];
    int held = 0;         // wave-uniform number of entries in the ring
    uint32_t mine = 0u;   // how many of them belong to this lane's query
    // one reservation per query, then every entry takes the next free slot of its query's share
    auto flush = [&]() {
#ifndef ETF_ABL
        wpos[w][lane] = mine ? atomicAdd(&o.cnt[ql], mine) : 0u;
        __builtin_amdgcn_wave_barrier();
        for (int i = lane; i < held; i += 64) {
            const uint64_t e = ring[w][i];
            const int owner = (int)((e >> 26) & 63u);
            const uint32_t pos = atomicAdd(&wpos[w][owner], 1u);
            const int64_t q = (int64_t)tile * QT + owner;
            if (pos < o.C) o.cand[q * o.C + pos] = (e & 0xFFFFFFFF00000000ull) | (e & 0x3FFFFFFull);
        }
        __builtin_amdgcn_wave_barrier();
#endif
        held = 0;
        mine = 0u;
    };
    float tauv = 0.f, best = __uint_as_float(0x7F800000u);
    if (MODE == OUT_FILTER) tauv = o.tau[ql];
    float ctx[DT];
#pragma unroll
    for (int s = 0; s < DT; ++s) ctx[s] = 0.f;

    // encoding number, tree-0 record and gather offsets of the item a lane owns in the chunk at `base`
    auto fetch = [&](int64_t base, uint32_t dw[NDW], uint32_t goff[TMAX], float &tm) {
        const bool live = base + lane < hi;
        const uint32_t e = live ? (MODE == OUT_FILTER ? (uint32_t)(base + lane) : map[base + lane]) : 0u;
        tm = (o.term && live) ? o.term[e] : 0.f;  // leaf term of the item this lane owns
#pragma unroll
        for (int i = 0; i < NDW; ++i) dw[i] = live ? codes0[(int64_t)e * NDW + i] : 0u;
#pragma unroll
        for (int t = 1; t < TMAX; ++t) goff[t] = live ? r.leaf_of[t][e] * (uint32_t)(QT * 4) : 0u;
    };
    // requests the rows of group g of a chunk (items past the end read row 0)
    constexpr int GV = NG1 > 0 ? GP : 1;
    auto gather = [&](const uint32_t goff[TMAX], int g, float v[GV][NV]) {
#pragma unroll
        for (int i = 0; i < GP; ++i) {
            const int src = g * GP + i;
#pragma unroll
            for (int t = 1; t < TMAX; ++t)
                v[i][t - 1] = buf_load(tabr[t], lane4, __builtin_amdgcn_readlane((int)goff[t], src));
        }
    };

    uint32_t my_dw[NDW], my_goff[TMAX], next_dw[NDW], next_goff[TMAX];
    float my_tm = 0.f, next_tm = 0.f;
    float va[GV][NV], vb[GV][NV];  // rows of the group being evaluated / of the group after it, alternating
    fetch(lo, my_dw, my_goff, my_tm);
    if (NG1 > 0) gather(my_goff, 0, va);
    for (int64_t base = lo; base < hi; base += 64) {
        const int cnt = uniform((int)min<int64_t>(64, hi - base));
        fetch(base + 64, next_dw, next_goff, next_tm);  // arrives while this chunk is evaluated
        ChunkMeta<DT> m;
        chunk_meta<DT, NDW, NL, UBT>(m, my_dw, codes0, base, lo, lane, cnt, pad, K, MODE == OUT_FILTER);
        // one group: evaluate its items with the rows in `cur`, and right after the first batch's lookups
        // are issued request the rows of the following group into `nxt`
        auto group = [&](int g, float cur[GV][NV], float nxt[GV][NV]) {
#pragma unroll
            for (int b = 0; b < NBAT; ++b) {
                const int s0 = g * GP + b * UBT;
                auto request = [&] {
                    if (NG1 > 0 && b == 0) {
                        if ((g + 1) * GP < 64) gather(my_goff, g + 1, nxt);
                        else gather(next_goff, 0, nxt);
                    }
                };
                if (s0 >= cnt) {
                    request();  // an empty group still passes the request for the rows on
                } else {
                    float d[UBT];
                    ctx_batch_any<DT, NL, UBT>(ctx, lutr, ldsb, lane4, m, s0, cnt, d, request);
                    {
#pragma unroll
                        for (int u = 0; u < UBT; ++u) {
#pragma unroll
                            for (int t = 1; t < TMAX; ++t) d[u] += (TMAX == 2 || t < r.T) ? cur[b * UBT + u][t - 1] : 0.f;
                            d[u] += __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_tm), min(s0 + u, 63)));
                        }
#pragma unroll
                        for (int u = 0; u < UBT; ++u) {
                            if (s0 + u >= cnt) break;
                            if (MODE == OUT_ALLPAIRS) tbuf[w][s0 + u][lane] = d[u];
                            else if (MODE == OUT_SAMPLE) best = fminf(best, d[u]);
                            else {
                                const bool pass = d[u] <= tauv;
                                const uint64_t mask = __ballot(pass);
                                if (mask != 0ull) {
                                    const int rank = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                                    __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                                    if (pass)
                                        ring[w][held + rank] = ((uint64_t)__float_as_uint(d[u]) << 32) |
                                                               ((uint32_t)lane << 26) | (uint32_t)(base + s0 + u);
                                    mine += pass ? 1u : 0u;
                                    held += __popcll(mask);
                                    if (held > RING - 64) flush();
                                }
                            }
                        }
                    }
                }
            }
        };
        // every group is visited, two per round so that the two row buffers swap roles without being copied
        for (int g = 0; g < NGRP; g += 2) {
            group(g, va, vb);
            if (NGRP > 1) group(g + 1, vb, va);
        }
        if (MODE == OUT_ALLPAIRS) {
            __builtin_amdgcn_wave_barrier();
            for (int qq = 0; qq < 64; ++qq) {
                const int64_t q = (int64_t)tile * QT + qq;
                if (q < o.nq && lane < cnt) o.dist[q * o.N + base + lane] = tbuf[w][lane][qq];
            }
            __builtin_amdgcn_wave_barrier();
        }
#pragma unroll
        for (int i = 0; i < NDW; ++i) my_dw[i] = next_dw[i];
#pragma unroll
        for (int t = 1; t < TMAX; ++t) my_goff[t] = next_goff[t];
        my_tm = next_tm;
    }
    if (MODE == OUT_FILTER) flush();
    if (MODE == OUT_SAMPLE) o.gmin[((int64_t)tile * o.ngroups + wv) * QT + lane] = best;
}

}  // namespace etf
