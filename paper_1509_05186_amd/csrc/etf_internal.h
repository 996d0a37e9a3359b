// Internal declarations shared by the host and device halves of the library.
#pragma once

#include <cstdint>
#include <cstdio>
#include <functional>
#include <string>
#include <vector>

#include "etf.h"

namespace etf {

constexpr int QT = 64;            // queries per tile: one partial-sum row is QT floats (256 bytes)
constexpr uint32_t NO_PARENT = 0xFFFFFFFFu;

// One internal level of one tree, in sorted (= breadth-first) order.
struct HostLevel {
    std::vector<uint8_t> code;     // chunk value of the node
    std::vector<uint32_t> parent;  // index into the previous level (NO_PARENT at level 1)
};

// All leaves of one tree whose own chunk is at the same level: equal record width.
struct HostBucket {
    int width = 0;                 // 1 + postfix length
    int stride = 0;                // record stride in bytes (width rounded up to 4)
    std::vector<uint8_t> codes;    // [n][stride], own chunk first, then the postfix, zero padded
    std::vector<uint32_t> parent;  // index into internal level (level-1), NO_PARENT for level 1
    std::vector<uint32_t> row;     // leaf number in sorted order = row of the tree's result table
    size_t size() const { return parent.size(); }
};

struct HostTree {
    int c0 = 0, D = 0;                      // covers chunks [c0, c0 + D)
    int64_t U = 0;                          // distinct sub-encodings = leaves
    std::vector<HostLevel> level;           // [D]   (entry l = level l+1; the last one is always empty)
    std::vector<HostBucket> bucket;         // [D]   (entry l = leaves at level l+1)
    std::vector<int64_t> nI, nL;            // [D]   internal nodes / leaves of level l+1 (the arrays above are empty
                                            //       when the index was built on the device)
    std::vector<uint32_t> leaf_of;          // [n_distinct] leaf row of every distinct full encoding (empty if T == 1)
    int rstride = 0;                        // bytes per record of `rec`: D rounded up to 1, 2, 4, 8 or 16, at least 4
    std::vector<uint8_t> rec;               // [U][rstride] the distinct sub-encodings in lexicographic order, zero padded
};

// smallest of 1, 2, 4, 8, 16 that is >= D: the unrolled depth of the register-context kernels
inline int depth_class(int D)
{
    int c = 1;
    while (c < D) c <<= 1;
    return c;
}

struct HostIndex {
    bool built = false;
    // Built on the device: the host holds the shape and the counts only, the image is already resident.
    bool device_built = false;
    int64_t n_sample_enc = 0, n_sample_pos = 0;  // entries of the two threshold samples
    int M = 0, K = 0, T = 0;
    int64_t N = 0, Nd = 0, max_dup = 0;
    std::vector<int32_t> chunk_begin;       // [T+1]
    std::vector<int32_t> order;             // [M] position j of the index's encodings holds input chunk order[j]
    std::vector<uint8_t> codes;             // [N][M] input order
    std::vector<int32_t> ids_in;            // [N] ids in input order
    std::vector<int32_t> ids_sorted;        // [N] ids in (encoding, id) order
    std::vector<uint32_t> ebegin;           // [Nd+1] range of ids_sorted of every distinct encoding
    std::vector<uint32_t> enc_of_pos;       // [N] distinct-encoding number of the n-th input vector
    std::vector<uint8_t> ecodes;            // [Nd][M] distinct encodings in sorted order
    std::vector<uint32_t> sample_enc;       // sorted distinct-encoding numbers of the threshold sample
    std::vector<uint32_t> sample_pos;       // input positions of the flat-mode threshold sample
    std::vector<uint8_t> sample_enc_codes;  // [n_sample_enc][M] the sampled encodings themselves, in sample order
    std::vector<uint8_t> sample_pos_codes;  // [n_sample_pos][M] likewise for the flat-mode sample
    // Leaf payload: one additive float32 term per vector, given before the build.  Vectors that share an encoding but
    // not the term are separate entries ("distinct encodings" below then means distinct (encoding, term) pairs).
    bool has_term = false;
    std::vector<float> eterm;               // [Nd] term of every entry
    std::vector<float> pterm;               // [N] term of every vector, input order
    int rstride0 = 0;
    std::vector<uint8_t> rec0;              // [Nd][rstride0] tree 0's chunks of every distinct encoding, zero padded
    std::vector<HostTree> tree;
};

// Device image: offsets (bytes) into the uploaded buffer.
struct DevTreeLayout {
    int64_t leaf_of = -1;
    int64_t rec = 0;
    int64_t icode[ETF_MAX_M], iparent[ETF_MAX_M];
    int64_t lcodes[ETF_MAX_M], lparent[ETF_MAX_M], lrow[ETF_MAX_M];
};

struct DevLayout {
    int64_t total = 0;
    int64_t codebooks = 0, codes = 0, ids_in = 0, ids_sorted = 0, ebegin = 0, enc_of_pos = 0, ecodes = 0,
            sample_enc = 0, sample_pos = 0, rec0 = 0, cb_centered = 0, cb_norm = 0, cb_mean = 0, sample_enc_codes = 0,
            sample_pos_codes = 0;
    int64_t eterm = -1, pterm = -1;         // only with a leaf payload
    std::vector<DevTreeLayout> tree;
};

// IVFADC index: the database as (cell of a coarse quantiser, encoding of the residual), sorted by (cell, encoding,
// id); equal (cell, encoding) pairs merged into one entry with an id range; list j = the entries of cell j.
struct IvfIndex {
    bool built = false;
    int Kc = 0;                         // cells
    std::vector<float> centroids;       // [Kc][d]
    std::vector<float> cnorm;           // [Kc] ||centroid||^2
    float cmax = 0.f;                   // largest ||centroid||, rounded up
    int64_t N = 0, Ne = 0;              // vectors, entries (distinct (cell, encoding) pairs)
    int64_t max_list = 0, max_dup = 0;  // most entries in one list, most vectors in one entry
    int64_t tree_lookups = 0;           // sum over the lists of the table lookups of the list's E-Tree (L1 + L2 + sumP)
    std::vector<uint32_t> lbegin;       // [Kc+1] range of entries of every cell
    std::vector<uint8_t> ecodes;        // [Ne][M]
    std::vector<float> eterm;           // [Ne] ||r||^2 + 2 <centroid, r>, r = the entry's reconstructed residual
    std::vector<uint32_t> ebegin;       // [Ne+1] range of ids_sorted of every entry
    std::vector<int32_t> ids_sorted;    // [N]
    int64_t o_centroids = 0, o_cnorm = 0, o_codebooks = 0, o_lbegin = 0, o_ecodes = 0, o_eterm = 0, o_ebegin = 0, o_ids = 0, total = 0;
    char *dev_base = nullptr;           // caller-owned buffer holding the image
};

struct Options {
    int64_t ws_cap_bytes = (int64_t)8 << 30;
    int64_t force_fallback = 0;
    int64_t sample_min = 32768;
    int64_t sample_scale = 120; // sample size = max(sample_min, sample_scale * sqrt(n))
    int64_t cand_cap = 0;
    int64_t traversal = 2;  // 0: distance context in registers, 1: level-synchronous kernels, 2: searches with all tables in LDS
    int lds16_context = 1;  // k_lds16 keeps a distance context of two levels (1) or looks every chunk up (0)
    int64_t lds_blocks = 0; // workgroups per sub-tile of queries in the LDS-resident search kernel (0: chosen by the library)
    int64_t metric = 0;     // 0: squared Euclidean distance (smallest first), 1: scalar product (largest first)
    int64_t lds_filter = 2; // main pass of the LDS-resident search: 0 float32 sums, 1 / 2 candidate filter in 32 / 16-bit fixed point
    int64_t encode_wide = 1;   // matrix-core encoder for groups of more than 64 dimensions: operands through LDS (1) or streamed per lane (0)
    int64_t encode_kernel = 0; // device encoder: 0 distance evaluations on the matrix cores, near-ties by the float32 rule; 1 the rule for every codeword
    int64_t ivf_coarse_kernel = 0; // IVFADC distances to the centroids: 0 matrix cores + the float32 rule near the w-th, 1 the rule for every cell
    int64_t ivf_coarse_tile = 1;   // the matrix-core distances with operands staged through LDS where the shape allows (1) or always streamed per lane (0)
    int64_t ivf_bound_factor = 16;  // IVFADC scan: the bound comes from the nearest lists that hold this many times k entries (0: from all lists)
    int64_t ivf_probe_slack = 1;   // factor on the error bound of the matrix-core distances (tests: more cells, or all, go through the rule)
    int64_t ivf_probe_cap = 0;     // cells the probe selection recomputes by the rule before it redoes the whole row (0: chosen by the library)
    int64_t lut_narrow_below = (int64_t)1 << 40; // (tile, group) pairs below which the table kernel runs as single-wave workgroups of 32 codewords (default: always)
    int64_t lut_kernel = 0; // 0: matrix cores (expanded form on centred vectors, small entries recomputed), 1: plain (a-b)^2 sums
};

// entries of the threshold sample for n candidates: the sample pass costs time in proportion to the sample, the
// candidates it lets through in inverse proportion, so the best size grows like the square root of n
int64_t sample_size(const Options &opt, int64_t n);

}  // namespace etf

struct etf_ctx {
    int device = -1;
    void *stream = nullptr;
    mutable std::string err;
    // quantiser
    int d = 0, M = 0, K = 0, ds = 0;
    std::vector<float> codebooks;           // [M][K][ds]
    std::vector<float> rotation;            // [d][d] row-major, or empty: the quantiser's space is y = rotation x (OPQ)
    int rot_d = 0;
    std::vector<float> rotation_t;          // the rotation transposed, staging for the device copy
    // for the matrix-core table build: codewords minus the group's mean codeword, rows padded to an even
    // length dsp; their squared norms; the means
    int dsp = 0;
    std::vector<float> cb_centered;         // [M][K][dsp]
    std::vector<float> cb_norm;             // [M][K]
    std::vector<float> cb_mean;             // [M][ds]
    // index
    etf::HostIndex idx;
    etf::IvfIndex ivf;
    etf::DevLayout lay;
    char *dev_base = nullptr;               // caller-owned buffer holding the device image
    etf::Options opt;
    std::vector<int32_t> next_order;        // chunk order of the next index build (empty: as given)
    std::vector<float> next_term;           // leaf payload of the next index build (empty: none)
    // diagnostics of the most recent search (device address inside the caller's workspace)
    void *last_flag_count = nullptr;
    // landing place of the small device-to-host copies of the device index build
    uint32_t build_scal[4] = {0, 0, 0, 0};
    // per-kernel timing: pairs of hipEvent_t (stored untyped so that host-only code need not see HIP)
    bool profile_on = false;
    bool no_alloc_call = false;     // inside etf_search_static: nothing that allocates (no new event pairs)
    struct Stamp { void *start, *stop; int cls; };
    std::vector<Stamp> stamps;      // recorded since the last read
    std::vector<Stamp> stamp_pool;  // events ready for reuse
};

namespace etf {

int fail(const etf_ctx *ctx, int code, const char *fmt, ...);
void compute_layout(etf_ctx *ctx);
// upper bound of the image bytes of an index over N vectors in T trees
int64_t image_bytes_bound(const etf_ctx *ctx, int64_t N, int T, const int32_t *chunk_begin);
void drop_index(etf_ctx *ctx);
void prepare_centered(etf_ctx *ctx);
// calls put(offset, pointer, bytes) for every array of the device image
void for_each_image_array(const etf_ctx *ctx, const std::function<void(int64_t, const void *, size_t)> &put);

// parallel for over [0, n) in contiguous slices, on up to `threads` std::threads
void parallel_slices(int64_t n, int threads, const std::function<void(int, int64_t, int64_t)> &fn);
int host_threads();

}  // namespace etf
