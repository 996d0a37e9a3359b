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
//     row: the query's Kc distances (not negative); pk: LDS for pow2(w) keys; probes, base: the query's w cells and
//     their distances.  Every thread of the workgroup of 256 calls it.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void ivf_probe_row(const float *row, int Kc, int w, uint64_t *pk, uint32_t *hist, uint32_t *sel_sh, uint32_t *s_n,
                                              int32_t *__restrict__ probes, float *__restrict__ base)
{
    // the w-th smallest distance, then, if more cells tie with it than are still needed, the largest cell number to take
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
    if (threadIdx.x == 0) *s_n = 0;
    __syncthreads();
    for (int c = threadIdx.x; c < Kc; c += 256) {
        const uint32_t v = __float_as_uint(row[c]);
        if (v < vstar || (v == vstar && (uint32_t)c <= cstar)) {
            const uint32_t pos = atomicAdd(s_n, 1u);
            if (pos < (uint32_t)w) pk[pos] = ((uint64_t)v << 16) | (uint32_t)c;
        }
    }
    __syncthreads();
    const int w2 = pow2_at_least(w);
    for (int i = w + threadIdx.x; i < w2; i += 256) pk[i] = ~0ull;
    __syncthreads();
    sort_u64(pk, w2);
    for (int i = threadIdx.x; i < w; i += 256) {
        probes[i] = (int32_t)(pk[i] & 0xFFFFu);
        base[i] = __uint_as_float((uint32_t)(pk[i] >> 16));
    }
}

//     grid (queries), block 256, dynamic LDS 8 * pow2(w) bytes; Kc <= 65536.
__global__ __launch_bounds__(256) void k_ivf_probe(const float *__restrict__ dist, int Kc, int w, int32_t *__restrict__ probes,
                                                   float *__restrict__ base)
{
    extern __shared__ uint64_t pk[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_n;
    __shared__ uint32_t sel_sh[8];
    const int64_t q = blockIdx.x;
    ivf_probe_row(dist + q * Kc, Kc, w, pk, hist, sel_sh, &s_n, probes + q * w, base + q * w);
}

// ------------------------------------------------------------------------------------------------
// The distance matrix of a batch of queries on the matrix cores, approximately, and without the query's own norm,
// which is the same along its row:  a[q][c] = ||c||^2 - 2 <q, c>  (v_mfma_f32_32x32x2_f32, A = queries, B =
// centroids, float32 in and out, operand layout as in k_lut_mfma: for a fixed accumulator register the lanes 0..31
// hold 32 consecutive cells of one query, a 128-byte piece of a row of the matrix).  The probed cells are not decided
// on these numbers: k_ivf_probe_mfma takes every cell that can be among the w nearest given the error of a[q][c] and
// decides among them by the float32 rule.
//     A wave owns 64 queries x 128 cells (2 x 4 accumulator blocks) and walks the dimensions 16 at a time (the two
//     k-slots of the instruction take the lower and the upper 8, so a lane reads 8 consecutive floats of each of
//     its six rows per block), the next block's operands in flight while the 64 instructions of this one run.
//     grid (ceil(nq / 128), ceil(Kc / 256)), block 256 (wave w: queries 64 (w & 1).., cells 128 (w >> 1)..).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_ivf_coarse_mfma(const float *__restrict__ x, int64_t n, int d, const float *__restrict__ cent,
                                                         const float *__restrict__ cnorm, int Kc, float *__restrict__ approx)
{
    const int lane = threadIdx.x & 63, w = uniform(threadIdx.x >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int64_t qb = (int64_t)blockIdx.x * 128 + (w & 1) * 64;
    const int cbase = (int)blockIdx.y * 256 + (w >> 1) * 128;
    if (qb >= n || cbase >= Kc) return;  // the whole wave: there is no barrier below
    const float *qrow[2], *crow[4];
    bool qlive[2], clive[4];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int64_t q = qb + rb * 32 + col;
        qlive[rb] = q < n;
        qrow[rb] = x + (qlive[rb] ? q : 0) * d;
    }
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        const int c = cbase + cb * 32 + col;
        clive[cb] = c < Kc;
        crow[cb] = cent + (int64_t)(clive[cb] ? c : 0) * d;
    }
    const bool wide = (d & 3) == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0 && (reinterpret_cast<uintptr_t>(cent) & 15) == 0;
    auto load8 = [&](const float *row, bool live, int j, float (&o)[8]) {
        if (wide && live && j + 8 <= d) {
            const float4 lo = *reinterpret_cast<const float4 *>(row + j), hi = *reinterpret_cast<const float4 *>(row + j + 4);
            o[0] = lo.x; o[1] = lo.y; o[2] = lo.z; o[3] = lo.w;
            o[4] = hi.x; o[5] = hi.y; o[6] = hi.z; o[7] = hi.w;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = (live && j + i < d) ? row[j + i] : 0.f;
        }
    };
    auto load_block = [&](int j0, float (&a)[2][8], float (&b)[4][8]) {
        const int j = j0 + 8 * half;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) load8(qrow[rb], qlive[rb], j, a[rb]);
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) load8(crow[cb], clive[cb], j, b[cb]);
    };
    floatx16 acc[2][4];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;
    auto multiply = [&](const float (&a)[2][8], const float (&b)[4][8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 4; ++cb) acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[rb][i], b[cb][i], acc[rb][cb], 0, 0, 0);
    };
    float a0[2][8], b0[4][8], a1[2][8], b1[4][8];
    if (wide && (d & 15) == 0) {
        // whole blocks of 16 dimensions, 16-byte loads: no branch between a load and its use, so that the wait before a
        // block's instructions covers that block's loads only and the next block's stay in flight.  Rows beyond the
        // batch or the cells read row 0 (their results are not stored); the block after the last is the last again.
        auto fetch = [&](int j0, float (&a)[2][8], float (&b)[4][8]) {
            const int j = min(j0, d - 16) + 8 * half;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const float4 lo = *reinterpret_cast<const float4 *>(qrow[rb] + j), hi = *reinterpret_cast<const float4 *>(qrow[rb] + j + 4);
                a[rb][0] = lo.x; a[rb][1] = lo.y; a[rb][2] = lo.z; a[rb][3] = lo.w;
                a[rb][4] = hi.x; a[rb][5] = hi.y; a[rb][6] = hi.z; a[rb][7] = hi.w;
            }
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
                const float4 lo = *reinterpret_cast<const float4 *>(crow[cb] + j), hi = *reinterpret_cast<const float4 *>(crow[cb] + j + 4);
                b[cb][0] = lo.x; b[cb][1] = lo.y; b[cb][2] = lo.z; b[cb][3] = lo.w;
                b[cb][4] = hi.x; b[cb][5] = hi.y; b[cb][6] = hi.z; b[cb][7] = hi.w;
            }
        };
        const int nblk = d >> 4;
        fetch(0, a0, b0);
        int blk = 0;
        for (; blk + 2 <= nblk; blk += 2) {
            fetch(16 * (blk + 1), a1, b1);
            multiply(a0, b0);
            fetch(16 * (blk + 2), a0, b0);
            multiply(a1, b1);
        }
        if (blk < nblk) multiply(a0, b0);
    } else {
        load_block(0, a0, b0);
        for (int j0 = 0; j0 < d; j0 += 32) {
            const bool second = j0 + 16 < d;
            if (second) load_block(j0 + 16, a1, b1);
            multiply(a0, b0);
            if (second) {
                if (j0 + 32 < d) load_block(j0 + 32, a0, b0);
                multiply(a1, b1);
            }
        }
    }
    float cn[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) cn[cb] = clive[cb] ? cnorm[cbase + cb * 32 + col] : 0.f;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t q = qb + rb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
            if (q >= n) continue;
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
                if (clive[cb]) approx[q * Kc + cbase + cb * 32 + col] = fmaf(-2.f, acc[rb][cb][r], cn[cb]);
        }
}

// ------------------------------------------------------------------------------------------------
// The same matrix with both operands staged through LDS, for d a multiple of 32 and 16-byte aligned rows: a workgroup
// owns 128 queries x 256 cells and walks the dimensions 32 at a time; the 384 rows of a stage (one 128-byte line each)
// are fetched with coalesced 16-byte loads, eight threads per row, held in registers while the previous stage is
// multiplied, and written to LDS rows of 36 floats (16 lanes reading one column of 16 rows hit 16 different bank
// quartets).  Same tiles per wave, same operand order and so the same values as k_ivf_coarse_mfma, whose per-lane
// loads of 16 bytes from 64 different lines keep the matrix cores waiting for the cache's tag look-ups.
//     grid (ceil(nq / 128), ceil(Kc / 256)), block 256, static LDS 384 * 36 * 4 bytes.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void k_ivf_coarse_tc(const float *__restrict__ x, int64_t n, int d, const float *__restrict__ cent,
                                                       const float *__restrict__ cnorm, int Kc, float *__restrict__ approx)
{
    constexpr int RS = 36;  // floats per LDS row
    __shared__ __attribute__((aligned(16))) float tile[384 * RS];
    const int t = threadIdx.x, lane = t & 63, w = uniform(t >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int64_t q0 = (int64_t)blockIdx.x * 128;
    const int c0 = (int)blockIdx.y * 256;
    // the rows this thread fetches: float4 number t + 256 i of the stage, i = 0..11, is piece t & 7 of row (t >> 3) +
    // 32 i; rows 0..127 (i < 4) are queries, 128..383 cells; rows beyond the batch or the cells read the last one (their
    // results are not stored)
    const int r0 = t >> 3, c4 = t & 7;
    // 32-bit offsets from the workgroup's first query and first cell (two workgroups share a compute unit if a wave
    // stays within 256 registers, 128 of them accumulators)
    const float *xq = x + q0 * d, *cc = cent + (int64_t)c0 * d;
    const int qrows = (int)min<int64_t>(128, n - q0), crows = min(256, Kc - c0);
    uint32_t off[12];
#pragma unroll
    for (int i = 0; i < 4; ++i) off[i] = (uint32_t)(min(r0 + 32 * i, qrows - 1) * d + 4 * c4);
#pragma unroll
    for (int i = 4; i < 12; ++i) off[i] = (uint32_t)(min(r0 + 32 * (i - 4), crows - 1) * d + 4 * c4);
    const int dst0 = r0 * RS + 4 * c4;  // LDS position of piece i: dst0 + 32 i RS
    floatx16 acc[2][4];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;
    const int arow = (w & 1) * 64, brow = 128 + (w >> 1) * 128;  // first LDS row of this wave's queries and cells
    typedef float vf4 __attribute__((ext_vector_type(4)));  // (an array of HIP's float4 structs stays in scratch memory here)
    vf4 st[12];
#pragma unroll
    for (int i = 0; i < 12; ++i) st[i] = *reinterpret_cast<const vf4 *>((i < 4 ? xq : cc) + off[i]);
    for (int j0 = 0; j0 < d; j0 += 32) {
        __syncthreads();  // the previous stage has been read
#pragma unroll
        for (int i = 0; i < 12; ++i) *reinterpret_cast<vf4 *>(tile + dst0 + 32 * i * RS) = st[i];
        __syncthreads();
        {
            const int jn = min(j0 + 32, d - 32);  // after the last stage: the last again (not used)
#pragma unroll
            for (int i = 0; i < 12; ++i) st[i] = *reinterpret_cast<const vf4 *>((i < 4 ? xq : cc) + off[i] + jn);
        }
        // the loads above are issued here, ahead of the stage's matrix instructions (left alone, the compiler sinks
        // them below those to save registers, and every stage then waits for the memory)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            const int j = 16 * blk + 8 * half;
            float a[2][8], b[4][8];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const float *p = tile + (arow + rb * 32 + col) * RS + j;
                const float4 lo = *reinterpret_cast<const float4 *>(p), hi = *reinterpret_cast<const float4 *>(p + 4);
                a[rb][0] = lo.x; a[rb][1] = lo.y; a[rb][2] = lo.z; a[rb][3] = lo.w;
                a[rb][4] = hi.x; a[rb][5] = hi.y; a[rb][6] = hi.z; a[rb][7] = hi.w;
            }
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
                const float *p = tile + (brow + cb * 32 + col) * RS + j;
                const float4 lo = *reinterpret_cast<const float4 *>(p), hi = *reinterpret_cast<const float4 *>(p + 4);
                b[cb][0] = lo.x; b[cb][1] = lo.y; b[cb][2] = lo.z; b[cb][3] = lo.w;
                b[cb][4] = hi.x; b[cb][5] = hi.y; b[cb][6] = hi.z; b[cb][7] = hi.w;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb)
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[rb][i], b[cb][i], acc[rb][cb], 0, 0, 0);
        }
    }
    const int64_t qb = q0 + (w & 1) * 64;
    const int cbase = c0 + (w >> 1) * 128;
    float cn[4];
    bool clive[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        clive[cb] = cbase + cb * 32 + col < Kc;
        cn[cb] = clive[cb] ? cnorm[cbase + cb * 32 + col] : 0.f;
    }
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t q = qb + rb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
            if (q >= n) continue;
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
                if (clive[cb]) approx[q * Kc + cbase + cb * 32 + col] = fmaf(-2.f, acc[rb][cb][r], cn[cb]);
        }
}

// One distance by the float32 rule (see k_ivf_coarse): q in LDS, c a centroid's row.
__device__ __forceinline__ float ivf_rule_distance(const float *q, const float *__restrict__ c, int d)
{
    float acc = 0.f;
    if ((d & 3) == 0 && (reinterpret_cast<uintptr_t>(c) & 15) == 0) {
#pragma unroll 8
        for (int j = 0; j < d; j += 4) {  // unrolled: the loads of eight steps are in flight together
            const float4 cv = *reinterpret_cast<const float4 *>(c + j);
            const float ce[4] = {cv.x, cv.y, cv.z, cv.w};
            {
#pragma clang fp contract(off)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float df = q[j + i] - ce[i];
                    const float p = df * df;
                    acc = acc + p;
                }
            }
        }
    } else {
        for (int j = 0; j < d; ++j) {
#pragma clang fp contract(off)
            const float df = q[j] - c[j];
            const float p = df * df;
            acc = acc + p;
        }
    }
    return acc;
}

// ------------------------------------------------------------------------------------------------
// Probe selection on the approximate matrix of k_ivf_coarse_mfma, with the result of the float32 rule.
//     With a = ||c||^2 - 2 <q, c> as computed there and r the rule's distance, |a + ||q||^2 - r| <= E for
//     E = (8 d + 16) 2^-24 (||q|| + max ||c||)^2: the centroid's norm, the contraction (d products, accumulated in
//     float32, taken at twice the unit roundoff), the last operation and the rule's own d + 2 roundings are each at
//     most their count times 2^-24 (||q|| + ||c||)^2, together (6 d + 7) of them.  So a cell among the w smallest
//     by the rule has a <= a_w + 2 E, a_w the w-th smallest a of the row, and so a <= t + 2 E for any t with at
//     least w cells at or below it (t: a bin edge of the row's range, see below).  Those cells are collected (a few
//     more than w), their distances computed by the rule, and the w smallest (distance, cell) of them are the probes:
//     the same cells, distances and order as k_ivf_coarse + k_ivf_probe give.  A row with more such cells than `cap`
//     (or none: a row with a NaN or an infinity) is recomputed by the rule in full, in place, and handled like there.
//     grid (queries), block 256, dynamic LDS ivf_probe_lds_bytes(w, cap, d); Kc <= 65536, cap >= w.
// ------------------------------------------------------------------------------------------------
__host__ __device__ inline int ivf_pow2(int n)
{
    int p = 1;
    while (p < n) p <<= 1;
    return p;
}
__host__ __device__ inline size_t ivf_probe_lds_bytes(int w, int cap, int d)
{
    (void)w;
    return (size_t)ivf_pow2(cap) * 8 + (size_t)cap * 4 + (size_t)((d + 3) & ~3) * 4;
}

// f(c, row[c]) for every cell of a row, by the 256 threads of a workgroup: eight 16-byte loads in flight per thread
// where the row allows them (a loop of single loads waits for the memory once per cell of the thread).
template <class F>
__device__ __forceinline__ void ivf_for_row(const float *__restrict__ row, int Kc, F f)
{
    if ((Kc & 3) == 0 && (reinterpret_cast<uintptr_t>(row) & 15) == 0) {
        const float4 *row4 = reinterpret_cast<const float4 *>(row);
        const int n4 = Kc >> 2;
        for (int i0 = 0; i0 < n4; i0 += 256 * 8) {
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * 256 + (int)threadIdx.x;
                v[u] = row4[min(i, n4 - 1)];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * 256 + (int)threadIdx.x;
                if (i < n4) {
                    f(4 * i, v[u].x);
                    f(4 * i + 1, v[u].y);
                    f(4 * i + 2, v[u].z);
                    f(4 * i + 3, v[u].w);
                }
            }
        }
    } else {
#pragma unroll 8
        for (int c = threadIdx.x; c < Kc; c += 256) f(c, row[c]);
    }
}

__global__ __launch_bounds__(256) void k_ivf_probe_mfma(const float *__restrict__ x, int d, const float *__restrict__ cent, float cmax, float slack,
                                                        float *__restrict__ approx, int Kc, int w, int cap,
                                                        int32_t *__restrict__ probes, float *__restrict__ base)
{
    extern __shared__ uint64_t pk[];
    __shared__ uint32_t hist[1024];
    __shared__ uint32_t s_n;
    __shared__ uint32_t sel_sh[8];
    __shared__ float s_red[4], s_lo[4], s_hi[4];
    const int cap2 = ivf_pow2(cap);
    int32_t *s_cell = reinterpret_cast<int32_t *>(pk + cap2);
    float *qs = reinterpret_cast<float *>(s_cell + cap);
    const int64_t q = blockIdx.x;
    float *row = approx + q * Kc;
    float part = 0.f;
    for (int j = threadIdx.x; j < d; j += 256) {
        const float v = x[q * d + j];
        qs[j] = v;
        part = fmaf(v, v, part);
    }
#pragma unroll
    for (int dlt = 32; dlt >= 1; dlt >>= 1) part += __shfl_xor(part, dlt);
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = part;
    if (threadIdx.x == 0) s_n = 0;
    __syncthreads();
    const float qq = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
    const float S = sqrtf(qq) * 1.001f + cmax;
    const float E2 = 2.f * (float)(8 * d + 16) * 5.9604645e-8f * 1.01f * S * S * slack;
    // A bound at or above the w-th smallest a of the row, without sorting anything: the row's range in 1024 equal bins,
    // the first bin at which the running count reaches w, its upper edge.  (A radix select on the float bits finds the
    // w-th itself, but its first digits are the same for nearly all cells: every count lands on one LDS word.)
    constexpr int NB = 1024;
    float lo = 3.402823466e+38f, hi = -3.402823466e+38f;
    ivf_for_row(row, Kc, [&](int, float v) {
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    });
#pragma unroll
    for (int dlt = 32; dlt >= 1; dlt >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, dlt));
        hi = fmaxf(hi, __shfl_xor(hi, dlt));
    }
    if ((threadIdx.x & 63) == 0) {
        s_lo[threadIdx.x >> 6] = lo;
        s_hi[threadIdx.x >> 6] = hi;
    }
    for (int i = threadIdx.x; i < NB; i += 256) hist[i] = 0u;
    __syncthreads();
    lo = fminf(fminf(s_lo[0], s_lo[1]), fminf(s_lo[2], s_lo[3]));
    hi = fmaxf(fmaxf(s_hi[0], s_hi[1]), fmaxf(s_hi[2], s_hi[3]));
    const float span = hi - lo;
    // false with a NaN or an infinity in the row, and for data so small that products of two values are subnormal (the
    // matrix instruction flushes those to zero, which the bound E does not cover): the rule then takes the whole row
    const bool usable = span >= 0.f && span < 3.0e38f && S * S > 1.0e-30f;
    const float scale = span > 0.f ? (float)NB / span : 0.f;
    auto bin_of = [&](float v) { return min(NB - 1, (int)((v - lo) * scale)); };
    if (usable) ivf_for_row(row, Kc, [&](int, float v) { atomicAdd(&hist[bin_of(v)], 1u); });
    __syncthreads();
    {
        // thread t owns bins 4t .. 4t+3; the running count before them by a scan over the threads
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        uint32_t h[4], own = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            h[i] = hist[4 * threadIdx.x + i];
            own += h[i];
        }
        uint32_t inc = own;
#pragma unroll
        for (int dlt = 1; dlt < 64; dlt <<= 1) {
            const uint32_t up = (uint32_t)__shfl_up((int)inc, dlt);
            if (lane >= dlt) inc += up;
        }
        if (lane == 63) sel_sh[wave] = inc;
        __syncthreads();
        for (int w2 = 0; w2 < wave; ++w2) inc += sel_sh[w2];
        uint32_t run = inc - own;
        const uint32_t need = (uint32_t)min(w, Kc);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (run < need && need <= run + h[i]) sel_sh[4] = (uint32_t)(4 * threadIdx.x + i);
            run += h[i];
        }
        if (threadIdx.x == 0 && !usable) sel_sh[4] = 0u;
        __syncthreads();
    }
    const float thr = usable ? lo + (float)(sel_sh[4] + 1u) * (span / (float)NB) + E2 : -3.402823466e+38f;
    if (usable)
        ivf_for_row(row, Kc, [&](int c, float v) {
            if (v <= thr) {
                const uint32_t pos = atomicAdd(&s_n, 1u);
                if (pos < (uint32_t)cap) s_cell[pos] = c;
            }
        });
    __syncthreads();
    const int ncand = (int)s_n;
    __syncthreads();
    if (ncand > cap || ncand < min(w, Kc)) {
        for (int c = threadIdx.x; c < Kc; c += 256) row[c] = ivf_rule_distance(qs, cent + (int64_t)c * d, d);
        __syncthreads();
        ivf_probe_row(row, Kc, w, pk, hist, sel_sh, &s_n, probes + q * w, base + q * w);
        return;
    }
    const int n2 = ivf_pow2(ncand);
    for (int i = threadIdx.x; i < n2; i += 256) {
        uint64_t key = ~0ull;
        if (i < ncand) {
            const int c = s_cell[i];
            key = ((uint64_t)__float_as_uint(ivf_rule_distance(qs, cent + (int64_t)c * d, d)) << 16) | (uint32_t)c;
        }
        pk[i] = key;
    }
    __syncthreads();
    sort_u64(pk, n2);
    for (int i = threadIdx.x; i < w; i += 256) {
        probes[q * w + i] = (int32_t)(pk[i] & 0xFFFFu);
        base[q * w + i] = __uint_as_float((uint32_t)(pk[i] >> 16));
    }
}

// ------------------------------------------------------------------------------------------------
// The probed lists of one query.
// ------------------------------------------------------------------------------------------------
struct IvfScanArgs {
    const float *lut;         // [nq][M][K] scalar products <q_m, codeword>
    const float *base;        // [nq][w] squared distances to the probed cells' centroids
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
    uint32_t bound_entries;   // scan: entries of the nearest lists that the bound is taken from (0: all lists)
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
// and no position has to be looked up among the lists.  f(entry, distance) runs for every entry of the first nlists
// lists.
// CM, CK: M and K as constants (the common shape, loops unrolled and table offsets immediate), or 0: taken from a.
template <int CM, int CK, class F>
__device__ __forceinline__ void ivf_walk_shape(const IvfScanArgs &a, const float *tab, const uint32_t *s_off, const uint32_t *s_lo,
                                               const float *s_base, int nlists, F f)
{
    const int M = CM ? CM : a.M, K = CK ? CK : a.K;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    for (int p = wave; p < nlists; p += nw) {
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
                                         const float *s_base, int nlists, F f)
{
    if (a.M == 8 && a.K == 256)
        ivf_walk_shape<8, 256>(a, tab, s_off, s_lo, s_base, nlists, f);
    else
        ivf_walk_shape<0, 0>(a, tab, s_off, s_lo, s_base, nlists, f);
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
        s_base[p] = a.base[q * a.w + p];
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
//     Pass 1 counts the vectors per distance bin (a histogram over the upper bits of the float) over the nearest
//     cells' lists, as many as together hold bound_entries entries, and finds the bin in which the running count
//     reaches k: its upper edge bounds the k-th distance.  Pass 2 evaluates the entries of all lists and appends
//     those at or below the bound to the query's candidate list, which k_select orders and expands.
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
    // The bound comes from the nearest cells alone: the first lists that together hold bound_entries entries (all, if
    // they do not).  The k-th smallest distance among part of the vectors is at or above the k-th among all.  Where
    // that bound lets more entries pass than the candidate list holds (a query whose neighbours sit in a farther
    // cell), the bound is taken again, from all lists.
    int nbound = a.w;
    if (a.bound_entries > 0) {
        int lo = 1, hi = a.w;  // smallest p with s_off[p] >= bound_entries
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_off[mid] >= a.bound_entries) hi = mid;
            else lo = mid + 1;
        }
        nbound = lo;
    }
    for (;;) {
        ivf_walk(a, tab, s_off, s_lo, s_base, nbound, [&](uint32_t e, float d) {
            atomicAdd(&hist[__float_as_uint(d) >> SH], min(a.ebegin[e + 1] - a.ebegin[e], (uint32_t)a.k));
        });
        __syncthreads();
        // the bin in which the running count of vectors reaches k (thread t owns bins [t * NB/256, (t+1) * NB/256))
        {
            constexpr int PER = NB / 256;
            uint32_t part = 0;
            for (int b = 0; b < PER; ++b) part += hist[threadIdx.x * PER + b];
            s_part[threadIdx.x] = part;
            if (threadIdx.x == 0) s_tau = 0x7F800000u;  // fewer than k vectors in the lists: everything passes
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
        ivf_walk(a, tab, s_off, s_lo, s_base, a.w, [&](uint32_t e, float d) {
            const uint32_t bits = __float_as_uint(d);
            if (bits <= tau) {
                const uint32_t pos = atomicAdd(&s_cnt, 1u);
                if (pos < a.C) a.cand[q * a.C + pos] = ((uint64_t)bits << 32) | e;
            }
        });
        __syncthreads();
        if (nbound == a.w || s_cnt <= a.C) break;
        __syncthreads();
        nbound = a.w;
        for (int i = threadIdx.x; i < NB; i += 256) hist[i] = 0;
        if (threadIdx.x == 0) s_cnt = 0;
        __syncthreads();
    }
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
    iv.o_cnorm = take((int64_t)iv.Kc * 4);
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
    int cap = 0;      // cells per query the probe selection recomputes by the float32 rule
    int64_t o_counter = 0, o_coarse = 0, o_probes = 0, o_base = 0, o_lut = 0, o_cnt = 0, o_flag = 0, o_cand = 0, total = 0;
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
    P.cap = ctx->opt.ivf_probe_cap ? (int)std::max<int64_t>(ctx->opt.ivf_probe_cap, w) : std::max(1024, 2 * w);
    const int64_t per_q = (int64_t)iv.Kc * 4 + (int64_t)w * 8 + (int64_t)ctx->M * ctx->K * 4 + 8 + C * 8;
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
    P.o_base = take(P.nqb * w * 4);
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
        ctx->ivf.cnorm.resize((size_t)Kc);
        double big = 0.0;
        for (int c = 0; c < Kc; ++c) {
            double t = 0.0;
            for (int j = 0; j < ctx->d; ++j) t += (double)centroids[(size_t)c * ctx->d + j] * (double)centroids[(size_t)c * ctx->d + j];
            ctx->ivf.cnorm[c] = (float)t;
            big = std::max(big, t);
        }
        ctx->ivf.cmax = (float)(std::sqrt(big) * 1.000001);
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
    HIP_TRY(ctx, hipMemcpyAsync(base + iv.o_cnorm, iv.cnorm.data(), iv.cnorm.size() * 4, hipMemcpyHostToDevice, st));
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
// the approximate distance matrix of n vectors: operands through LDS where the rows allow it
static void ivf_launch_coarse(etf_ctx *ctx, const float *x, int64_t n, const float *cent, const float *cnorm, float *matrix)
{
    const int d = ctx->d, Kc = ctx->ivf.Kc;
    const dim3 grid((unsigned)((n + 127) / 128), (unsigned)((Kc + 255) / 256));
    hipStream_t st = (hipStream_t)ctx->stream;
    if ((d & 31) == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0 && (reinterpret_cast<uintptr_t>(cent) & 15) == 0 && ctx->opt.ivf_coarse_tile != 0)
        hipLaunchKernelGGL(k_ivf_coarse_tc, grid, dim3(256), 0, st, x, n, d, cent, cnorm, Kc, matrix);
    else
        hipLaunchKernelGGL(k_ivf_coarse_mfma, grid, dim3(256), 0, st, x, n, d, cent, cnorm, Kc, matrix);
}

// vectors per batch of the coarse assignment: their distance matrix stays within 256 MiB
static int64_t ivf_assign_batch(const etf_ctx *ctx, int64_t n)
{
    const int64_t by_bytes = ((int64_t)256 << 20) / ((int64_t)ctx->ivf.Kc * 4);
    return std::max<int64_t>(1, std::min<int64_t>(n, std::max<int64_t>(256, by_bytes)));
}

extern "C" int64_t etf_ivf_assign_workspace_bytes(const etf_ctx *ctx, int64_t n)
{
    if (!ctx) return ETF_EINVAL;
    if (ctx->codebooks.empty() || ctx->ivf.Kc == 0) return fail(ctx, ETF_ESTATE, "need codebooks and etf_ivf_set_coarse first");
    if (n < 0) return fail(ctx, ETF_EINVAL, "n is negative");
    const int64_t nb = ivf_assign_batch(ctx, n);
    return ivf_al((int64_t)ctx->ivf.Kc * ctx->d * 4) + ivf_al((int64_t)ctx->ivf.Kc * 4) + ivf_al(nb * ctx->ivf.Kc * 4) + ivf_al(nb * 4) +
           ivf_al(etf_encode_workspace_bytes(ctx)) + ivf_al(n * ctx->d * 4);
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
    const int d = ctx->d;
    const int64_t nb = ivf_assign_batch(ctx, n);
    char *w = (char *)ws;
    float *cent = (float *)w;
    w += ivf_al((int64_t)iv.Kc * d * 4);
    float *cnorm = (float *)w;
    w += ivf_al((int64_t)iv.Kc * 4);
    float *matrix = (float *)w;
    w += ivf_al(nb * iv.Kc * 4);
    float *nearest = (float *)w;
    w += ivf_al(nb * 4);
    char *enc_ws = w;
    const int64_t enc_bytes = ivf_al(etf_encode_workspace_bytes(ctx));
    float *res = (float *)(enc_ws + enc_bytes);
    HIP_TRY(ctx, hipMemcpyAsync(cent, iv.centroids.data(), iv.centroids.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipMemcpyAsync(cnorm, iv.cnorm.data(), iv.cnorm.size() * 4, hipMemcpyHostToDevice, st));
    {
        ProfScope prof(ctx, ETF_K_ENCODE);
        if (ctx->opt.ivf_coarse_kernel == 0) {
            // the cell of a vector is its one probed cell: smallest (distance, cell) by the float32 rule
            const int cap = 1024;
            const size_t lds_probe = ivf_probe_lds_bytes(1, cap, d);
            if (lds_probe > 150 * 1024) return fail(ctx, ETF_EINVAL, "d=%d needs %zu bytes of LDS for the cell selection", d, lds_probe);
            rc = set_lds(ctx, k_ivf_probe_mfma, lds_probe);
            if (rc) return rc;
            for (int64_t v0 = 0; v0 < n; v0 += nb) {
                const int64_t nv = std::min<int64_t>(nb, n - v0);
                ivf_launch_coarse(ctx, x + v0 * d, nv, cent, cnorm, matrix);
                LAUNCH_CHECK(ctx, "k_ivf_coarse_mfma");
                hipLaunchKernelGGL(k_ivf_probe_mfma, dim3((unsigned)nv), dim3(256), lds_probe, st, x + v0 * d, d, cent, iv.cmax,
                                   (float)ctx->opt.ivf_probe_slack, matrix, iv.Kc, 1, cap, cells_out + v0, nearest);
                LAUNCH_CHECK(ctx, "k_ivf_probe_mfma");
            }
        } else {
            hipLaunchKernelGGL(k_ivf_coarse<true>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x, n, d, cent, iv.Kc, nullptr, cells_out, iv.Kc);
            LAUNCH_CHECK(ctx, "k_ivf_coarse");
        }
        hipLaunchKernelGGL(k_ivf_residual, dim3((unsigned)((n * d + 255) / 256)), dim3(256), 0, st, x, n, d, cent, cells_out, res);
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
    const size_t lds_probe = ivf_probe_lds_bytes(w, P.cap, d);
    if (lds_probe > 150 * 1024) return fail(ctx, ETF_EINVAL, "w=%d with d=%d needs %zu bytes of LDS for the probe selection", w, d, lds_probe);
    rc = set_lds(ctx, k_ivf_probe_mfma, lds_probe);
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
        float *pbase = reinterpret_cast<float *>(wsp + P.o_base);
        {
            ProfScope prof(ctx, ETF_K_IVF_COARSE);
            if (ctx->opt.ivf_coarse_kernel == 0) {
                const float *cnorm = reinterpret_cast<const float *>(img + iv.o_cnorm);
                ivf_launch_coarse(ctx, qb, nq, cent, cnorm, coarse);
                LAUNCH_CHECK(ctx, "k_ivf_coarse_mfma");
                hipLaunchKernelGGL(k_ivf_probe_mfma, dim3((unsigned)nq), dim3(256), lds_probe, st, qb, d, cent, iv.cmax, (float)ctx->opt.ivf_probe_slack, coarse, iv.Kc, w, P.cap, probes,
                                   pbase);
                LAUNCH_CHECK(ctx, "k_ivf_probe_mfma");
            } else {
                // about 2048 workgroups: the centroids in slices of whole tiles of 32
                const int64_t qblocks = (nq + 255) / 256;
                int64_t slices = std::max<int64_t>(1, std::min<int64_t>((iv.Kc + 31) / 32, 2048 / qblocks));
                const int cslice = (int)(((iv.Kc + slices - 1) / slices + 31) / 32 * 32);
                slices = (iv.Kc + cslice - 1) / cslice;
                hipLaunchKernelGGL(k_ivf_coarse<false>, dim3((unsigned)qblocks, (unsigned)slices), dim3(256), 0, st, qb, nq, d, cent, iv.Kc, coarse,
                                   nullptr, cslice);
                LAUNCH_CHECK(ctx, "k_ivf_coarse");
                hipLaunchKernelGGL(k_ivf_probe, dim3((unsigned)nq), dim3(256), (size_t)pow2_at_least_host(w) * 8, st, coarse, iv.Kc, w, probes, pbase);
                LAUNCH_CHECK(ctx, "k_ivf_probe");
            }
        }
        {
            // tables of scalar products <q_m, codeword>, one set per query, shared by all cells
            ProfScope prof(ctx, ETF_K_LUT);
            const int64_t tiles = (nq + QT - 1) / QT;
            hipLaunchKernelGGL((k_lut_mfma<true, 2>), dim3((unsigned)tiles, (unsigned)M), dim3(256), 0, st, qb, nq, (int64_t)0, d, M, K, cbd, nullptr,
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
        a.base = pbase;
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
        a.bound_entries = (uint32_t)std::min<int64_t>((int64_t)ctx->opt.ivf_bound_factor * k, 0x7FFFFFFF);
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
