/*
 * etf.h -- C ABI of the E-Tree / E-Forest asymmetric-distance library for MI355X (gfx950).
 *
 * The library computes, for a batch of uncompressed float32 queries, the
 * asymmetric distances (ADC) to a database of product-quantised vectors
 * (M one-byte codes per vector, K <= 256 codewords per group), either flat
 * (paper: Related Work, Eq. 1 and the paragraph after it: "M table lookups and
 * M-1 additions") or through an Encoding Tree / Encoding Forest (paper:
 * sections "Encoding Tree", "Constructing Encoding Tree", "Distance Computation
 * with Hierarchical Memory Structure", "Encoding Forests"), in which the partial
 * sum of a shared code prefix is computed once.
 *
 * Conventions
 *   - Every function returns ETF_OK (0) or a negative ETF_E* code; nothing
 *     throws or aborts across this boundary.  etf_last_error() gives a text for
 *     the most recent failure on a context.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device
 *     memory of the context's GPU (for example torch tensor data_ptr()).  The
 *     caller owns every buffer.  The library keeps no reference to a buffer
 *     after a call returns, with one exception: the index buffer given to
 *     etf_index_upload() must stay alive and unmodified until etf_destroy() or
 *     the next etf_index_upload().
 *   - Device entry points enqueue their work on the context's stream and return
 *     without synchronising; results are ready when the stream is.  They
 *     validate arguments on the host first and launch nothing on error.
 *   - Distances are squared Euclidean distances.  Codes are 0-based bytes.
 *     Arrays are row-major, dense, in the index order written in the comments.
 *   - Limits: 1 <= M <= ETF_MAX_M, d % M == 0, 1 <= K <= 256, 1 <= N < 2^31,
 *     1 <= T <= M, 1 <= k <= ETF_MAX_TOPK.
 */
#ifndef ETF_H
#define ETF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ETF_MAX_M 16       /* code chunks per vector */
#define ETF_MAX_TOPK 1024  /* largest k of etf_search */

enum {
    ETF_OK = 0,
    ETF_EINVAL = -1, /* bad argument (null pointer, shape, range)             */
    ETF_ESTATE = -2, /* call order: e.g. search before index upload           */
    ETF_ENOMEM = -3, /* host allocation failed, or caller's buffer too small  */
    ETF_EHIP = -4,   /* a HIP runtime call failed                             */
    ETF_ENOGPU = -5  /* device entry point called on a host-only context      */
};

/* How distances are evaluated (results agree up to float32 summation order). */
enum {
    ETF_MODE_FLAT = 0,   /* every encoding: M lookups (the paper's ADC baseline)            */
    ETF_MODE_TREE = 1,   /* single Encoding Tree; the index must have been built with T = 1 */
    ETF_MODE_FOREST = 2  /* Encoding Forest: T per-tree partial results summed per encoding */
};

typedef struct etf_ctx etf_ctx; /* opaque */

/* Tree statistics (paper: "Statistics of Encoding Tree").  Levels are 1-based in
 * the text and stored 0-based here: entry [t][l] is level l+1 of tree t. */
typedef struct etf_stats {
    int32_t M, K, T;
    int32_t chunk_begin[ETF_MAX_M + 1];    /* tree t covers chunks [chunk_begin[t], chunk_begin[t+1]) */
    int64_t N;                             /* database vectors                                          */
    int64_t n_distinct;                    /* distinct full encodings                                   */
    int64_t max_dup;                       /* most vectors sharing one full encoding                    */
    int64_t nI[ETF_MAX_M][ETF_MAX_M];      /* internal nodes per level                                  */
    int64_t nL[ETF_MAX_M][ETF_MAX_M];      /* leaves whose own chunk is at that level                   */
    int64_t L1[ETF_MAX_M];                 /* internal nodes per tree                                   */
    int64_t L2[ETF_MAX_M];                 /* leaves per tree (= distinct sub-encodings)                */
    int64_t sumP[ETF_MAX_M];               /* total postfix length over the leaves                      */
    int64_t lookups[ETF_MAX_M];            /* table lookups of one traversal: L1 + L2 + sumP            */
    int64_t paper_bytes[ETF_MAX_M];        /* 4N + 2(L1+L2) + sumP (Hierarchical Memory Structure)      */
    int64_t device_bytes;                  /* size of the level-ordered device image                    */
    int32_t chunk_order[ETF_MAX_M];        /* position j of the index's encodings holds input chunk [j] */
} etf_stats;

/* ---- context ------------------------------------------------------------ */

/* Creates a context.  device >= 0 selects the HIP device that all device entry
 * points of this context use; device < 0 makes a host-only context (PQ
 * training, encoding, index build and statistics work; device entry points
 * return ETF_ENOGPU).  hip_stream is a hipStream_t (NULL = the default stream);
 * it is borrowed, not owned. */
int etf_create(etf_ctx **out, int device, void *hip_stream);
void etf_destroy(etf_ctx *ctx);
int etf_set_stream(etf_ctx *ctx, void *hip_stream);
const char *etf_strerror(int code);
const char *etf_last_error(const etf_ctx *ctx);

/* Tunables, by name.  Known names:
 *   "ws_cap_bytes"    upper bound the library aims at for the workspace (it
 *                     processes queries in batches to stay below it)
 *   "force_fallback"  1: etf_search answers every query with the exact
 *                     whole-database selection kernel (testing)
 *   "sample_min" / "sample_scale"   size of the sample that bounds the k-th distance (drawn by
 *                     etf_index_build): max(sample_min, sample_scale * sqrt(n)), n = number of distinct
 *                     encodings (of vectors in flat mode); defaults 32768 and 120
 *   "cand_cap"        per-query candidate capacity (0 = derived from k)
 *   "lds16_context"   1 (default): the 16-bit filter pass keeps the paper's Distance Context for the first two levels
 *                     (a wave whose lane groups all stay inside their two-chunk prefix skips those two lookups).
 *                     0: every chunk of every encoding is looked up (same results; measured 3 to 6 % slower at M = 8
 *                     and 4 % faster at M = 16, where the two skipped reads leave a bank-conflict pattern behind)
 *   "lds_blocks"      workgroups per sub-tile of queries in the LDS-resident kernels (0 = chosen by the
 *                     library from the number of sub-tiles and items; for experiments)
 *   "metric"          0 (default): squared Euclidean distance.  1: scalar product (the paper notes, after
 *                     Eq. 1 and in its conclusion, that tables of scalar products serve the same
 *                     machinery): etf_lut_build gives lut[q][m][c] = <queries[q] group m, codeword c>,
 *                     etf_adc gives dist[q][n] = <q, reconstruction of vector n> as the plain sum of the
 *                     table entries, etf_search returns the k LARGEST scalar products, descending, ties by
 *                     ascending id, out_dist holding the products.  Searches order candidates as
 *                     B(q) - <q, x> with B(q) the sum of every group's largest table entry, so a returned
 *                     product carries a rounding error of a few units in the last place of B(q), not of
 *                     the product itself.  Takes effect on the next call; the index does not depend on it
 *   "lut_kernel"      0 (default): lookup tables on the matrix cores, as ||q'||^2 - 2 q'.c' + ||c'||^2
 *                     on vectors shifted by the group's mean codeword; entries below a quarter of
 *                     ||q'||^2 + ||c'||^2, where that form cancels, are recomputed as plain sums.
 *                     1: every entry as a plain float32 sum of (q - c)^2
 *   "lut_narrow_below"  the matrix-core table kernel runs as workgroups of one wave and 32 codewords when the batch
 *                     has fewer (tile of 64 queries, group) pairs than this (default: always), else as workgroups
 *                     of four waves and 256 codewords; same tables either way
 *   "traversal"       how trees are walked.
 *                     0: depth-first leaf order with the distance context in registers, per-tree
 *                     result tables in device memory for trees 1 .. T-1;
 *                     1: level-synchronous kernels over the level arrays (partial sums of internal
 *                     nodes in device memory);
 *                     2 (default): every table slice of a group of queries is kept in LDS; searches
 *                     walk the sorted encodings with a short distance context per lane group,
 *                     etf_adc evaluates the input positions in order; no result tables at all (built
 *                     for M in {4, 8, 16} and equal trees of 1, 2 or a multiple of 4 chunks); every other
 *                     shape runs as 0.
 *                     0 and 1 add the chunks left to right and return identical bits; 2 adds the
 *                     chunks of every group of four in pairs and agrees with them to rounding.
 *   "encode_kernel"   etf_pq_encode_device (and the residual encoding of etf_ivf_assign_device).  0 (default): the
 *                     K distance evaluations of every (vector, group) on the matrix cores as ||c||^2 - 2 x.c;
 *                     where the smallest is not clearly below the second smallest (by twice a bound on the
 *                     rounding of either form) the float32 rule is evaluated for all K codewords.  1: the float32
 *                     rule for every codeword (needs d/M <= 128).  Both return the same codes, bit for bit
 *   "encode_wide"     1 (default): groups of more than 64 dimensions with aligned rows take the matrix-core kernel
 *                     that stages both operands through LDS; 0: the general one (operands streamed per lane)
 *   "ivf_coarse_kernel"  etf_ivf_search, distances between queries and centroids.  0 (default): all of them on the
 *                     matrix cores as ||c||^2 - 2 q.c; the cells that can be among the w nearest, given a bound on
 *                     the rounding of that form and of the float32 rule, are then evaluated by the rule, which
 *                     decides.  1: the rule for every cell.  Both give the same probed cells, distances and order
 *   "ivf_coarse_tile" 1 (default): that contraction stages its operands through LDS where d is a multiple of 32 and the
 *                     rows are 16-byte aligned; 0: every lane streams its own operand rows (the kernel for other d)
 *   "ivf_probe_cap"   most cells per query evaluated by the rule before the whole row is (0 = default: max(1024, 2 w);
 *                     never below w), "ivf_probe_slack" a factor >= 1 on that rounding bound (default 1): both for tests
 *   "ivf_bound_factor"  etf_ivf_search, scan of the probed lists: the bound on the k-th distance is taken from the
 *                     nearest cells' lists that together hold this many times k entries (default 16), and from all
 *                     probed lists if that bound lets more entries pass than the candidate list holds; 0: always
 *                     from all lists.  The result does not depend on it
 *   "lds_filter"      the main pass of searches with traversal 2, which looks at every distinct encoding and only has
 *                     to decide which of them can be among the k nearest.
 *                     0: float32 sums of the table entries, compared with the query's bound (from the sample).
 *                     1: 32-bit fixed point: every table entry is scaled so that the query's bound becomes 2^27,
 *                     truncated, and cut off at 2^28; sums of entries are integer additions, three operands per
 *                     instruction, compared with the bound rounded up.
 *                     2 (default): 16-bit fixed point, for M = 8 and M = 16 at K = 256 without leaf payload (other
 *                     shapes run as 0): the bound becomes 2^12 (M = 8) or 2^11 (M = 16), entries are truncated and
 *                     cut off at twice that, so that a sum of M entries fits 16 bits; twice the queries share a
 *                     workgroup's tables, a 16-byte LDS read serves 8 queries, and the sums are 32-bit additions of
 *                     two packed entries each, three operands per instruction.
 *                     With 1 and 2 no encoding whose float32 distance is at or below the bound is lost (entries are
 *                     rounded down, the bound up); of the survivors, those within the rounding of the k-th smallest
 *                     sum get their distance recomputed as the float32 sum of the float32 table entries, and those
 *                     distances are what is ordered and returned.  The recomputation adds in the order of the float32
 *                     pass, so ids and distances are those of 0, bit for bit.
 * Returns ETF_EINVAL for an unknown name or a value out of range. */
int etf_set_option(etf_ctx *ctx, const char *name, int64_t value);

/* ---- product quantiser, host side (paper: Introduction, Related Work) ---- */

/* Lloyd k-means per dimension group on x [n][d] (host): K codewords of d/M
 * dimensions per group, `iters` iterations, initial codewords drawn from the
 * training rows with a generator seeded by `seed`.  Replaces any codebooks and
 * any index held by the context. */
int etf_pq_train(etf_ctx *ctx, const float *x, int64_t n, int d, int M, int K, int iters, uint64_t seed);
/* Installs codebooks cb [M][K][d/M] (host) trained elsewhere. */
int etf_pq_set_codebooks(etf_ctx *ctx, const float *cb, int d, int M, int K);
/* Copies the codebooks to cb_out [M][K][d/M] (host). */
int etf_pq_get_codebooks(const etf_ctx *ctx, float *cb_out);
/* codes_out[i][m] = index of the codeword of group m nearest to x[i]'s group-m
 * sub-vector (lowest index on ties).  x [n][d] host, codes_out [n][M] host. */
int etf_pq_encode(const etf_ctx *ctx, const float *x, int64_t n, uint8_t *codes_out);

/* ---- rotation in front of the quantiser (paper, Related Work: Optimized Product Quantization is among the
 *      quantisers whose codes the tree stores; a preprocessing step, not part of the distance computation) --------
 * The quantiser then works on y = R x: train on, encode and query with rotated vectors; for an orthogonal R the
 * distances are those of the original space.  Rotating is explicit: the library never rotates behind a call.
 * etf_pq_set_rotation: R [d][d] host, row-major, finite (NULL clears; d need not match codebooks that are set until
 *   vectors are rotated).  etf_pq_get_rotation: R_out [d][d].
 * etf_rotate (host) / etf_rotate_device (device pointers, enqueued on the context's stream; ws: device, 256-byte
 *   aligned, at least etf_rotate_workspace_bytes; not in place): out[i] = R x[i] for n vectors of d floats, every
 *   component accumulated in double over the dimensions in ascending order and rounded to float once; host and
 *   device return the same bits.
 * etf_opq_train: the non-parametric alternation on x [n][d] (host): `rounds` times { rotate the training set,
 *   etf_pq_train on it with `iters` Lloyd iterations, replace R by the orthogonal matrix nearest to
 *   sum decode(encode(R x)) x^T }, then a last training on the rotated set; starts from the rotation that is set (the
 *   identity if none, or if its size is not d) and leaves rotation and codebooks set.  rounds = 0 is etf_pq_train
 *   behind the current rotation.  Cost per round: O(n d^2 + d^3 * tens) on the host. */
int etf_pq_set_rotation(etf_ctx *ctx, const float *R, int d);
int etf_pq_get_rotation(const etf_ctx *ctx, float *R_out);
int etf_rotate(const etf_ctx *ctx, const float *x, int64_t n, float *out);
int64_t etf_rotate_workspace_bytes(const etf_ctx *ctx);
int etf_rotate_device(etf_ctx *ctx, const float *x, int64_t n, float *out, void *ws, int64_t ws_bytes);
int etf_opq_train(etf_ctx *ctx, const float *x, int64_t n, int d, int M, int K, int iters, int rounds, uint64_t seed);

/* ---- index build, host side (paper: Algorithm 1, Hierarchical Memory Structure) ---- */

/* Sorts the encodings lexicographically and builds T encoding trees.
 *   codes        [N][M] host, every byte < K
 *   ids          [N] host, non-negative, or NULL for ids 0..N-1.  Reported by etf_search.
 *   T            number of trees (1 = Encoding Tree, >1 = Encoding Forest)
 *   chunk_begin  [T+1] host, strictly increasing from 0 to M; NULL = equal
 *                contiguous groups (T must divide M)
 * In each tree a node below which a single distinct (sub-)encoding remains is a
 * leaf carrying the rest of that encoding as postfix; vectors with equal
 * encodings share one leaf.  Requires codebooks (for M and K). */
int etf_index_build(etf_ctx *ctx, const uint8_t *codes, int64_t N, const int32_t *ids, int T,
                    const int32_t *chunk_begin);
int etf_index_stats(const etf_ctx *ctx, etf_stats *out);

/* Leaf payload (paper, Experiments: an additive quantiser's extra term, quantised to one byte, stored on the leaf
 * node).  The next etf_index_build attaches the additive term term[n] (host, [N] float32, non-negative and finite) to
 * vector n; every distance the library then reports for that vector (etf_adc, etf_search, all modes and traversals)
 * is the sum of its table entries plus its term, the term added last.  Vectors that share an encoding but not the
 * term are separate leaves (separate entries of the index; n_distinct counts (encoding, term) pairs), vectors that
 * share both share one.  etf_index_set_leaf_bytes is the one-byte form: term = offset + scale * bytes[n], evaluated
 * once in float32 with a fused multiply-add.  A NULL pointer clears a pending payload; a payload belongs to one build.
 * etf_index_build_device does not take a payload (ETF_ESTATE while one is pending); scalar-product searches (option
 * "metric" = 1) add the term to the shifted value they order by, i.e. they return the k largest <q, x> - term. */
int etf_index_set_leaf_term(etf_ctx *ctx, const float *term, int64_t N);
int etf_index_set_leaf_bytes(etf_ctx *ctx, const uint8_t *bytes, int64_t N, float scale, float offset);

/* Chunk order (paper: "Encoding Chunk Ordering": which chunk sits at which level decides how many
 * prefixes are shared; and the forest's choice of which chunks form a tree).
 * etf_index_set_chunk_order: the next etf_index_build / etf_index_build_device stores, at position j of
 * every encoding, the input's chunk order[j] ([M] host, a permutation of 0..M-1; NULL = as given), and
 * chunk_begin then cuts the reordered positions into trees.  Distances, ids and all-pairs outputs keep
 * their meaning (queries and codebooks stay in the quantiser's order; the library reorders its lookup
 * tables to match); float32 sums may differ in the last bits because the order of additions follows the
 * positions.  The array `codes` of the device image holds the reordered encodings.
 * etf_suggest_chunk_order: a greedy order for the given codes ([N][M] host) and tree shape: tree after
 * tree, level after level, the remaining chunk that splits the tree's prefixes so far into the fewest
 * distinct prefixes (evaluated on at most 2^18 evenly spaced vectors); if that order does not save
 * lookups on those vectors, the given order is returned.  order_out [M]; lookups_given /
 * lookups_order (either may be NULL) receive the table lookups of one traversal, L1 + L2 + sumP summed
 * over the trees, of those vectors' index in the given and in the suggested order. */
int etf_index_set_chunk_order(etf_ctx *ctx, const int32_t *order);
/* etf_suggest_partition: which chunks form a tree.  For T trees it tries the cuts of the M positions into T contiguous
 * groups (all of them while there are at most 64, otherwise a descent from the equal cut, one boundary one position at a
 * time), each with etf_suggest_chunk_order's greedy order for that cut, on at most 2^16 evenly spaced vectors of `codes`
 * ([N][M] host), and returns the cut and order whose index needs the fewest table lookups per traversal:
 * chunk_begin_out [T+1], order_out [M] (for etf_index_set_chunk_order and etf_index_build); lookups_equal /
 * lookups_best (either may be NULL): the lookups on those vectors with the equal cut and with the returned one. */
int etf_suggest_partition(const etf_ctx *ctx, const uint8_t *codes, int64_t N, int T, int32_t *chunk_begin_out,
                          int32_t *order_out, int64_t *lookups_equal, int64_t *lookups_best);
int etf_suggest_chunk_order(const etf_ctx *ctx, const uint8_t *codes, int64_t N, int T, const int32_t *chunk_begin,
                            int32_t *order_out, int64_t *lookups_given, int64_t *lookups_order);
/* Bytes of device memory the built index needs. */
int64_t etf_index_device_bytes(const etf_ctx *ctx);
/* Copies the index (and the codebooks) into dev_buf (device, 256-byte aligned,
 * at least etf_index_device_bytes()).  Synchronises the stream before returning. */
int etf_index_upload(etf_ctx *ctx, void *dev_buf, int64_t bytes);

/* Where each array of the device image starts (byte offsets into the buffer of
 * etf_index_upload / etf_index_export; -1 = array not present).  Entry [t][l] is
 * level l+1 of tree t.
 *   codebooks   float [M][K][d/M]
 *   codes       u8  [N][M]       encodings in input order (flat mode)
 *   ids_in      i32 [N]          ids in input order
 *   ids_sorted  i32 [N]          ids ordered by (encoding, id)
 *   ebegin      u32 [n_distinct+1]  range of ids_sorted held by every distinct encoding
 *   enc_of_pos  u32 [N]          distinct-encoding number of the n-th input vector
 *   ecodes      u8  [n_distinct][M]  distinct encodings in lexicographic order
 *   sample_enc  u32 [n_sample_enc]   numbers of distinct encodings used to bound the k-th distance (random order),
 *                                    drawn through vectors: an encoding appears in proportion to the number of
 *                                    vectors that have it, repeats dropped
 *   sample_pos  u32 [n_sample_pos]   input positions used for the same purpose in flat mode
 *   sample_enc_codes / sample_pos_codes  u8 [n_sample_*][M]  the encodings of those samples, in sample order
 *   leaf_of[t]  u32 [n_distinct] leaf (row of tree t's result table) of every distinct
 *                                encoding; absent when T = 1 (the identity)
 *   rec0 / trec[t]   the sorted distinct (sub-)encodings again as records of 4, 8 or 16 bytes:
 *                            the depth-first leaf sequence of each tree, walked by the kernels that
 *                            keep the distance context in registers.  A tree of D chunks uses the
 *                            last D of the first P bytes of a record, P = D rounded up to 1, 2, 4, 8
 *                            or 16; all other bytes are zero
 *   icode / iparent [t][l]   internal nodes of a level in lexicographic (= breadth-first)
 *                            order: chunk value (u8) and index of the parent in level l (u32;
 *                            0xFFFFFFFF at level 1)
 *   lcodes / lparent / lrow [t][l]   leaves whose own chunk is at this level: records of
 *                            lstride bytes (own chunk, postfix, zero padding), parent index
 *                            in the internal level above, and result-table row            */
typedef struct etf_layout {
    int64_t total;
    int64_t codebooks, codes, ids_in, ids_sorted, ebegin, enc_of_pos, ecodes, sample_enc, sample_pos;
    int64_t n_sample_enc, n_sample_pos;
    int64_t leaf_of[ETF_MAX_M];
    int64_t icode[ETF_MAX_M][ETF_MAX_M], iparent[ETF_MAX_M][ETF_MAX_M];
    int64_t lcodes[ETF_MAX_M][ETF_MAX_M], lparent[ETF_MAX_M][ETF_MAX_M], lrow[ETF_MAX_M][ETF_MAX_M];
    int32_t lstride[ETF_MAX_M][ETF_MAX_M];
    int64_t rec0;                  /* u8 [n_distinct][rec0_stride]: tree 0's chunks of every distinct encoding */
    int32_t rec0_stride;
    int64_t trec[ETF_MAX_M];       /* u8 [L2 of tree t][trec_stride[t]]: the tree's leaves as plain records     */
    int32_t trec_stride[ETF_MAX_M];
    int64_t cb_centered;           /* float [M][K][cb_row]: codewords minus their group's mean codeword, zero padded */
    int64_t cb_norm;               /* float [M][K]: squared norms of those                                            */
    int64_t cb_mean;               /* float [M][d/M]: the mean codeword of every group                                */
    int64_t sample_enc_codes;      /* u8 [n_sample_enc][M]: ecodes rows of sample_enc, in sample order               */
    int64_t sample_pos_codes;      /* u8 [n_sample_pos][M]: codes rows of sample_pos, in sample order                */
    int32_t cb_row;
    int64_t eterm;                 /* float [n_distinct]: leaf term of every entry; -1 without a leaf payload         */
    int64_t pterm;                 /* float [N]: leaf term of every vector, input order; -1 without a leaf payload    */
} etf_layout;
int etf_index_layout(const etf_ctx *ctx, etf_layout *out);
/* Writes the device image to host memory (at least etf_index_device_bytes()): the
 * same bytes etf_index_upload copies to the GPU.  For saving or inspecting an index. */
int etf_index_export(const etf_ctx *ctx, void *host_buf, int64_t bytes);

/* ---- device side -------------------------------------------------------- */

/* Device encoder (paper: Introduction, product quantisation; complexity O(dKN) in
 * "Efficient Encoding Tree Construction").  Same result definition as
 * etf_pq_encode, decided in float32: every squared distance is the sum of its
 * (x - c)^2 terms in dimension order, one rounding per operation, lowest index on
 * ties.  x [n][d] device, codes_out [n][M] device; ws is device scratch of at least
 * etf_encode_workspace_bytes() bytes (256-byte aligned) that receives the codebooks;
 * the copy is enqueued on the context's stream from the context's host copy.
 * Option "encode_kernel" = 1 needs d/M <= 128 (ETF_EINVAL otherwise).  n = 0 is allowed. */
int64_t etf_encode_workspace_bytes(const etf_ctx *ctx);
int etf_pq_encode_device(etf_ctx *ctx, const float *x, int64_t n, uint8_t *codes_out, void *ws, int64_t ws_bytes);

/* Index build on the device (paper: "Efficient Encoding Tree Construction":
 * Algorithm 1 — the in-place lexicographic sort of the encoded dataset and the
 * tree from the common prefixes of consecutive sorted encodings — built in
 * parallel, as the closing remark of that section suggests: radix sort, then per
 * level one flag pass over the neighbours' common prefix lengths, a prefix sum that
 * numbers the nodes, and a scatter).  Same arguments and the same index as
 * etf_index_build, except:
 *   codes   [N][M] u8, DEVICE (for example the output of etf_pq_encode_device)
 *   ids     [N] non-negative, DEVICE, or NULL for ids = position
 *   chunk_begin  host, as in etf_index_build
 *   image   device, 256-byte aligned; receives the index and becomes the resident
 *           index of the context: no etf_index_upload, and the buffer must stay
 *           alive and unmodified like the one given to etf_index_upload.
 *           *image_bytes of etf_index_build_device_bytes() always suffices (every
 *           array at its largest: as many distinct encodings as vectors); the
 *           build uses etf_index_device_bytes() of it, known afterwards, and
 *           returns ETF_ENOMEM as soon as an array does not fit a smaller buffer
 *   workspace  device scratch, 256-byte aligned, at least *workspace_bytes; free
 *           to reuse when the call returns
 * The image has the layout of etf_index_layout, array for array what
 * etf_index_build + etf_index_upload produce, except the two threshold samples
 * (one row from each of n_sample equal strata here; which rows are sampled
 * changes no result).  etf_index_export and etf_index_upload return ETF_ESTATE:
 * the host holds no copy.
 * Synchronises the stream several times (the counts that size the arrays come
 * back to the host).  On any error the context holds no index. */
int etf_index_build_device_bytes(const etf_ctx *ctx, int64_t N, int T, const int32_t *chunk_begin,
                                 int64_t *image_bytes, int64_t *workspace_bytes);
int etf_index_build_device(etf_ctx *ctx, const uint8_t *codes, int64_t N, const int32_t *ids, int T,
                           const int32_t *chunk_begin, void *image, int64_t image_bytes, void *workspace,
                           int64_t workspace_bytes);

/* Workspace (device bytes) that etf_adc / etf_search need for Q queries in the
 * given mode (k is ignored by etf_adc: pass 0).  Negative = error code. */
int64_t etf_workspace_bytes(const etf_ctx *ctx, int64_t Q, int k, int mode);

/* Precomputed distance tables (paper: Eq. 1, first term, on each group's own
 * dimensions): lut[q][m][c] = || queries[q] group m  -  codeword c of group m ||^2.
 *   queries [Q][d] device, lut [Q][M][K] device. */
int etf_lut_build(etf_ctx *ctx, const float *queries, int64_t Q, float *lut);

/* All-pairs ADC: dist[q][n] = distance between query q and the n-th vector given
 * to etf_index_build (input order, not id value).
 *   queries [Q][d] device, dist [Q][N] device, ws device workspace of ws_bytes. */
int etf_adc(etf_ctx *ctx, const float *queries, int64_t Q, int mode, float *dist, void *ws, int64_t ws_bytes);

/* k nearest encodings per query: out_ids [Q][k] (the ids given at build),
 * out_dist [Q][k], ascending by (distance, id).  k <= N. */
int etf_search(etf_ctx *ctx, const float *queries, int64_t Q, int k, int mode, int32_t *out_ids,
               float *out_dist, void *ws, int64_t ws_bytes);

/* etf_search for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results (bit for
 * bit) and same kernels as etf_search, but the workspace is a fixed array of ETF_STATIC_SCRATCH_BYTES in the
 * library's device image, one per GPU, held until the process ends; the call allocates nothing (no
 * hipMalloc / hipFree, no event creation: etf_profile_enable has no effect on it).  Queries go through in
 * batches of tiles of 64 that fit the array; a search whose single tile does not fit (very large candidate
 * capacity: flat mode over heavily repeated encodings, a large "cand_cap") returns ETF_ENOMEM and launches
 * nothing.  Every call on a GPU uses that GPU's one array (the counters in it are cleared by the call
 * itself): calls that overlap on one GPU, from any context or stream, race; so does etf_last_fallback_count
 * against a later call.  etf_static_scratch_bytes() returns the array's size. */
#define ETF_STATIC_SCRATCH_BYTES (64 << 20)
int64_t etf_static_scratch_bytes(void);
int etf_search_static(etf_ctx *ctx, const float *queries, int64_t Q, int k, int mode, int32_t *out_ids,
                      float *out_dist);

/* Number of queries of the most recent etf_search on this context that were
 * answered by the exact whole-database selection kernel instead of the
 * threshold-filtered path (diagnostic).  Synchronises the stream.  The count
 * lives in the first word of that search's workspace: the workspace must still
 * be allocated and unchanged when this is called (the one other place where
 * the library refers to a caller's buffer after a call).  ETF_ESTATE if no
 * search has run since the index was built or uploaded. */
int etf_last_fallback_count(etf_ctx *ctx, int64_t *out);

/* ---- IVFADC on the merged, sorted encodings -------------------------------- */

/* The paper's application experiment ("Application on related algorithms", Table 1): an inverted file with a coarse
 * quantiser of K' cells, the residual x - centroid product-quantised with the context's codebooks, w probed cells
 * per query, the ADC of every probed list on its Encoding Tree's leaf sequence: the entries of a cell sorted by
 * encoding, equal encodings merged into one entry with an id range.  A stored vector's distance
 *     || q - c - r ||^2  =  || q - c ||^2  +  ( ||r||^2 + 2 <c, r> )  -  2 <q, r>
 * (c its centroid, r its reconstructed residual) is evaluated as: the first term from the probe selection (by the
 * float32 rule below), the second a float32 constant stored with the entry (the "extra information stored on the leaf node" of the paper's
 * Experiments section), the third a sum of M entries of scalar-product tables that depend on the query only.
 * The terms cancel when q is close to the stored vector: a returned distance carries a rounding error of a few
 * 2^-24 of || q - c ||^2 + ||r||^2 + 2 |<q - c, r>| + 2 |<c, r>|, not of the distance itself.
 * Decisions that pick an integer (a vector's cell, a query's probed cells, a residual's codewords) are taken in
 * float32: a squared distance is the sum of its (a - b)^2 terms in dimension order, one rounding per operation,
 * lowest index on ties.
 *
 * etf_ivf_set_coarse   installs centroids [cells][d] (host; 1 <= cells <= 65536); needs the codebooks (for d).
 *                      Drops any IVF index of the context.
 * etf_ivf_assign_device  database side on the device: cells_out[i] = nearest centroid of x[i], codes_out[i] = the
 *                      encoding of x[i] - centroid (float32 subtraction).  x [n][d], cells_out [n], codes_out [n][M]
 *                      device; ws device scratch of etf_ivf_assign_workspace_bytes(n), 256-byte aligned.
 * etf_ivf_build        builds the index from cells [N] and codes [N][M] (host; for example the output of
 *                      etf_ivf_assign_device, or a reference's), ids [N] non-negative or NULL for 0..N-1.
 * etf_ivf_upload       copies it into dev_buf (device, 256-byte aligned, etf_ivf_device_bytes()), which must stay
 *                      alive and unmodified while searches run.  Synchronises the stream.
 * etf_ivf_search       per query the k nearest vectors among those of its w probed cells (the w nearest centroids),
 *                      ascending by (distance, id): out_ids [Q][k], out_dist [Q][k] device; a query whose probed
 *                      cells hold fewer than k vectors gets id -1 and +inf beyond them.  1 <= w <= min(cells, 4096).
 *                      Enqueues on the context's stream; etf_last_fallback_count applies. */
typedef struct etf_ivf_stats_t {
    int32_t cells;
    int64_t N, entries;          /* vectors; distinct (cell, encoding) pairs                                    */
    int64_t max_list, max_dup;   /* most entries in one cell; most vectors in one entry                         */
    int64_t tree_lookups;        /* table lookups of one traversal of every cell's Encoding Tree: L1 + L2 + sumP */
    int64_t flat_lookups;        /* N * M: what plain ADC over the same lists costs                              */
    int64_t device_bytes;
} etf_ivf_stats_t;
int etf_ivf_set_coarse(etf_ctx *ctx, const float *centroids, int cells);
int64_t etf_ivf_assign_workspace_bytes(const etf_ctx *ctx, int64_t n);
int etf_ivf_assign_device(etf_ctx *ctx, const float *x, int64_t n, int32_t *cells_out, uint8_t *codes_out, void *ws,
                          int64_t ws_bytes);
int etf_ivf_build(etf_ctx *ctx, const int32_t *cells, const uint8_t *codes, int64_t N, const int32_t *ids);
int etf_ivf_stats(const etf_ctx *ctx, etf_ivf_stats_t *out);
int64_t etf_ivf_device_bytes(const etf_ctx *ctx);
int etf_ivf_upload(etf_ctx *ctx, void *dev_buf, int64_t bytes);
int64_t etf_ivf_workspace_bytes(const etf_ctx *ctx, int64_t Q, int k, int w);
int etf_ivf_search(etf_ctx *ctx, const float *queries, int64_t Q, int k, int w, int32_t *out_ids, float *out_dist,
                   void *ws, int64_t ws_bytes);

/* ---- per-kernel timing (for benchmarks) ---------------------------------- */

/* Kernel classes of the hot path, in launch order. */
enum {
    ETF_K_LUT = 0,      /* lookup-table build                                 */
    ETF_K_LEVEL = 1,    /* internal tree levels                               */
    ETF_K_LEAF = 2,     /* leaf buckets                                       */
    ETF_K_FLAT = 3,     /* flat ADC (filter or all-pairs output)              */
    ETF_K_REDUCE = 4,   /* forest reduction (filter or all-pairs output)      */
    ETF_K_TAU = 5,      /* per-query bound from the sample                    */
    ETF_K_SELECT = 6,   /* final top-k selection                              */
    ETF_K_EXACT = 7,    /* exact whole-database selection                     */
    ETF_K_SAMPLE = 8,   /* distances of the bound's sample (flat or reduction) */
    ETF_K_LDS = 9,      /* tree / forest search with every table slice in LDS  */
    ETF_K_ENCODE = 10,  /* device encoder (and the coarse assignment of etf_ivf_assign_device) */
    ETF_K_IVF_COARSE = 11, /* IVFADC: distances to the centroids and probe selection */
    ETF_K_IVF_SCAN = 12,   /* IVFADC: scan of the probed lists                        */
    ETF_K_LDS16 = 13,      /* tree / forest candidate filter on 16-bit tables in LDS  */
    ETF_K_COUNT = 14
};
/* on != 0: every later kernel launch of this context is bracketed by a pair of
 * HIP events on the context's stream. */
int etf_profile_enable(etf_ctx *ctx, int on);
/* Synchronises the stream, then returns per class the summed kernel time in
 * milliseconds (ms[ETF_K_COUNT]) and the number of launches
 * (launches[ETF_K_COUNT]) since the last read, and resets both. */
int etf_profile_read(etf_ctx *ctx, double *ms, int64_t *launches);

/* ---- memory bandwidth probes (for benchmarks) ---------------------------- */

/* Plain streaming kernels over caller-owned device buffers, enqueued on the context's stream: the rates this
 * card's memory delivers, which a benchmark quotes as ceilings beside the traversal kernels (not part of the
 * paper's method).  a, b: device, 256-byte aligned; bytes: a multiple of 256, at least 64 KiB; b must hold at
 * least 16 KiB in every kind.
 *   ETF_PROBE_READ   reads `bytes` of a front to back (b receives one word per workgroup)
 *   ETF_PROBE_WRITE  writes `bytes` of a
 *   ETF_PROBE_COPY   copies `bytes` from a to b
 *   ETF_PROBE_ROWS   reads a as rows of 256 bytes, one wave per row, every row once, in a scattered order
 *   ETF_PROBE_LDS    no device memory traffic: 1024 workgroups of 16 waves read `bytes` in total from LDS, 16 bytes
 *                    per lane and instruction, conflict-free (a unused; b receives one word per workgroup)
 *   ETF_PROBE_LDS_SCATTER  the same with the access pattern of the table lookups: groups of four lanes read
 *                    64-byte rows at hashed positions (bank conflicts as they fall)
 *   ETF_PROBE_VALU_F32 / _ADD3 / _PK16  no memory traffic either: the rate at which the vector units issue one kind of
 *                    instruction (v_add_f32; v_add3_u32; v_pk_add_u16) from eight independent chains per lane; here
 *                    `bytes` is the number of lane instructions to execute in total, rounded down to a multiple of
 *                    2048 x 256 x 64 (a unused; b receives one word per workgroup, 8 KiB)
 *   ETF_PROBE_MFMA_F32  the rate of the float32 matrix instruction (v_mfma_f32_32x32x2_f32, eight independent
 *                    accumulator blocks per wave, four waves per workgroup); `bytes` is the number of floating-point
 *                    operations to execute in total, rounded down to a multiple of 2048 x 4 x 32 x 4096 (a unused; b as above) */
enum {
    ETF_PROBE_READ = 0, ETF_PROBE_WRITE = 1, ETF_PROBE_COPY = 2, ETF_PROBE_ROWS = 3, ETF_PROBE_LDS = 4, ETF_PROBE_LDS_SCATTER = 5,
    ETF_PROBE_VALU_F32 = 6, ETF_PROBE_VALU_ADD3 = 7, ETF_PROBE_VALU_PK16 = 8, ETF_PROBE_MFMA_F32 = 9
};
int etf_probe_bandwidth(etf_ctx *ctx, int kind, void *a, void *b, int64_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* ETF_H */
