// Argument blocks shared by the host-side C ABI (knn_api.cpp) and the kernels
// (knn_kernels.hip).  Plain structs passed by value at launch.
#ifndef KNN_DEVICE_H_
#define KNN_DEVICE_H_

#include <hip/hip_runtime_api.h>
#include <stdint.h>

#ifndef KNN_DC
#define KNN_DC 16          // coordinates staged through LDS per step
#endif
#define KNN_MAX_KCAP 128   // largest list capacity (>= KNN_MAX_K of the ABI)
#define KNN_FIN_MAX 2048   // most keys per query finalize_rows can merge (S * kcap)
#define KNN_QRES_MAX_D 256 // largest padded d whose query operands are kept resident in registers
#define KNN_TILE 128       // queries per workgroup tile == references per tile
#ifndef KNN_FOLD_NR
#define KNN_FOLD_NR 64      // fold kernel: references per tile (accumulators per lane), multiple of 16
#endif

namespace knn {

typedef unsigned long long u64;
constexpr u64 KEY_INF = ~0ull;

struct PrepArgs {
    const float *X;    // [n, d]
    int64_t n;
    int32_t d, dpad, metric;
    float *q_out;      // [n, dpad] query-side copy (scaled by -2 or -1/|x|), or null
    float *r_out;      // [n, dpad] reference-side copy (x or x/|x|), or null
    float *c_out;      // [n_cpad]  c_j, +inf beyond n, or null
    int64_t n_cpad;
    float *s_out;      // [n] squared norms, or null
    uint32_t *b_out;   // [n] per-query bound shared by the slices of the reference range: set to "none yet", or null
    const float *mu;   // [dpad] or null: subtracted from every row first (squared Euclidean only: no distance changes)
};

// split-precision experiment: a row as two bf16 pieces (see prep_split)
struct SplitPrepArgs {
    const float *X;    // [n, d]
    int64_t n;
    int32_t d, dpad;
    float scale;       // a power of two (-2: query side, 1: reference side)
    uint32_t *out;     // [n, dpad] words: per chunk of 32 coordinates 32 hi pieces, then 32 lo pieces
    float *c_out;      // [n_cpad] |x|^2, +inf beyond n, or null
    int64_t n_cpad;
    float *s_out;      // [n] |x|^2, or null
    uint32_t *b_out;   // [n] per-query bound shared by the slices: set to "none yet", or null
    const float *mu;   // [dpad] or null: subtracted from every row before the scaling
};

struct TileArgs {
    const float *Qp;   // [nq, ldq]
    const float *Rp;   // [nr, ldr]
    const float *cR;   // [n_rtiles * 128]
    u64 *lists;        // [S, nq_pad, kcap]
    uint32_t *bound;   // [nq] smallest k-th-best distance any slice has reached (order-preserving bits), or null (S == 1)
    int64_t ldq, ldr;
    int64_t nq, nr, nq_pad;
    int64_t self_offset;
    int32_t dpad, k, kcap;
    int32_t n_qtiles, n_rtiles, S, rt_per_split;
    const int32_t *nq_dev;    // knn_tiles_qreg<.., SUBSET> only: device word holding the number of queries (<= nq)
    const int32_t *self_rows; // ... and per query the reference index that is the query itself, or -1
};

// fold kernel (distances that are not inner products): lane = query, references from
// scalar registers
struct FoldArgs {
    const float *Qpk;  // queries packed by tile of 64 rows: [ceil(nq/64)][dpad/4][64 rows][4 coordinates]
    const float *Rpk;  // references packed by tile: [ceil(nr/NR)][dpad/4][NR rows][4 coordinates], NR = KNN_FOLD_NR
    u64 *lists;        // [S, nq_pad, kcap]
    uint32_t *bound;   // [nq_pad] smallest k-th-best distance any slice has reached, order-preserving bits
    int64_t nq, nr, nq_pad;
    int64_t self_offset;
    int64_t refs_per_split; // multiple of KNN_FOLD_NR
    int32_t dpad, k, kcap, metric, S;
};

// the fold with its distances written out (two-phase form)
struct FoldDistArgs {
    const float *Qpk;  // as FoldArgs
    const float *Rpk;
    float *D;          // [ceil(nq/128)*128, ldd]
    float *Dm;         // mirrored values: D, or the buffer of the transposed block (see DistArgs)
    float *M, *Mm;     // chunk minima of D and of the mirrored values (see DistArgs), or null
    int64_t ldm;
    int64_t ldd;
    int64_t nq, nr;
    int64_t self_offset;
    int64_t n_tiles;   // reference tiles of KNN_FOLD_NR rows
    int32_t dpad, metric;
    int32_t chunk;     // reference tiles per workgroup
    int32_t n_chunks;  // workgroups per block of query groups (those past the end leave at once)
    int32_t n_qblocks; // blocks of 4 query groups (256 rows)
};

struct PackArgs {
    const float *X;    // [n, d]
    float *Xpk;        // [ceil(n/NR)][dpad/4][NR][4]; zero where the source has no value
    int64_t n;
    int32_t d, dpad, rows_per_tile;
    uint32_t *bound;   // optional [n]: set to "no bound yet" (all ones) on the way
};

// What a Phase-1 kernel covers: all of the block (direct values only); the triangle of a square
// block from the diagonal on, mirrored into the same buffer; or all of a rectangle of two
// different row panels, mirrored into the buffer of the transposed block.
enum { DIST_FULL = 0, DIST_TRIANGLE = 1, DIST_RECT_MIRROR = 2 };

// Phase 1 of the two-phase organisation: the matrix of p(q, j), written out
struct DistArgs {
    const float *Qp;   // [nq, ldq]
    const float *Rp;   // [nr, ldr]
    const float *cR;   // [>= n_rt * 64], +inf past the end
    const float *cQ;   // [nq] c of the queries (symmetric mode; the same array as cR)
    float *D;          // [ceil(nq/128)*128, ldd]
    float *Dm;         // where the mirrored values go: D itself (triangle of one square block), or the
                       // buffer of the transposed block [ceil(nr/128)*128, ldd] (rectangle of two row panels)
    float *M;          // per row and chunk of 32 columns the smallest value stored in D, [rows of D, ldm], or
                       // null: lets select_rows skip the chunks that cannot matter
    float *Mm;         // the same for the mirrored values (rows of Dm)
    const float *tauQ; // [nq] or null: value of the k-th entry of the list a query row already has (+inf if it
                       // is short of k).  A chunk of 32 columns whose minimum is above it cannot change the
                       // list, select_rows will pass over it (it reads M first): it is not stored.
                       // knn_dist_qreg only, and only together with M / Mm.
    const float *tauR; // [nr] or null: the same for the rows the mirrored values go to
    int64_t ldq, ldr, ldd, ldm;
    int64_t nq, nr;
    int64_t self_offset;
    int32_t dpad;
    int32_t n_rt;      // reference tiles of 64 rows (knn_dist_stream: of 128 rows)
    int32_t chunk;     // reference tiles per workgroup
    int32_t n_chunks;  // workgroups per query tile (those past the end of their sweep leave at once)
    int32_t n_qtiles;  // query tiles of 128 rows
};

// symmetric schedule: one launch = one round of block pairs (round < 0: the diagonal blocks)
struct PairArgs {
    const float *Qp;   // [n, ldq] query-side copy
    const float *Rp;   // [n, ldr] reference-side rows
    const float *cR;   // [ceil(n/128)*128]
    const float *cmax; // device scalar: max_j c_j
    u64 *lists;        // [ceil(n/128)*128, kcap]
    int64_t ldq, ldr, n;
    int32_t dpad, k, kcap, metric;
    int32_t B;         // rows per block, multiple of 128
    int32_t NB;        // number of blocks
    int32_t NBp;       // NB rounded up to even
    int32_t round;     // 0 .. NBp-2, or -1
};

enum { FIN_RESCORE_SQ = 0, FIN_RESCORE_COS = 1, FIN_ADD_SQ = 2, FIN_ADD_ONE = 3, FIN_SELECT = 4, FIN_RESCORE_HEL = 5,
       FIN_RESCORE_L1 = 6, FIN_RESCORE_LINF = 7, FIN_RESCORE_KL = 8, FIN_ADD_SQ_SIGNED = 9 };

struct FinArgs {
    const u64 *lists;
    const float *Q;    // original query rows  [nq, d]   (re-score); FIN_SELECT: the matrix, row pitch nr, or null
    const float *R;    // original references  [nr, d]
    const float *sq;   // [nq] squared norms of the queries
    int32_t *idx;      // [nq, k]
    float *dist;       // [nq, k]
    int64_t nq, nq_pad;
    int64_t nr;        // number of reference rows (indices outside [0, nr) are never dereferenced)
    int32_t d, k, kcap, S, mode, vec4;
    // Filter-and-refine (split-precision experiment; FIN_RESCORE_SQ only): the lists were selected on
    // approximate values p~ with |p~ - p| <= err_a |q| + err_b for every reference.  The first
    // `krs` (> k) entries are priced exactly and the k best of them reported; the row is CERTIFIED
    // when the bound proves that no reference outside those krs can be among the true k nearest,
    // and counted in *uncert otherwise.  krs == 0: none of this.
    int32_t krs;
    int32_t all_kept;  // 1: there are no more than krs references in all, nothing was left out
    const float *cmax; // device scalar max_j |r_j|^2 (err_a, err_b are relative to its root / to it)
    double err_a, err_b;
    int32_t *uncert;   // device counter of rows not certified, or null
    int32_t *unc_rows; // [unc_cap] the first unc_cap of them, in order of arrival, or null
    int32_t unc_cap;
    // Second pass over a compacted subset of the queries (the rows listed in unc_rows by an earlier
    // call): block q serves query row row_map[q] and leaves if q >= *nq_dev.  null: block q is row q.
    const int32_t *row_map;
    const int32_t *nq_dev;
};

// split-precision plan, between its two passes: the rows the filter could not certify, scaled and
// padded for the fp32 kernel
struct GatherArgs {
    const float *Q;         // [nq, d] original query rows
    const int32_t *rows;    // [cap] uncertified rows (the first min(*count, cap) are valid)
    const int32_t *count;   // device word: rows not certified by the first pass
    float *q_out;           // [cap, dpad] = -2 Q[rows[i]], zero padded
    int32_t *self_out;      // [cap] self_offset + rows[i], or -1
    uint32_t *b_out;        // [cap] shared bound of the slices: "none yet"
    int32_t *n_out;         // device word: min(*count, cap), the size of the subset
    int32_t *left_out;      // device word or null: rows still unproven after the second pass, max(0, *count - cap)
    const float *mu;        // [dpad] or null: subtracted from the row before the scaling
    int64_t self_offset;
    int32_t d, dpad, cap;
};

// batched partial sort of a materialised matrix
struct SelectArgs {
    const float *A;    // [m, lda]
    u64 *lists;        // [S, m, kcap]
    int64_t m, n, lda;
    int64_t seg;       // columns per segment (multiple of 1024)
    int32_t k, kcap, S, vec4;
    int32_t resume;    // 0: lists start empty; 1: they hold the result of earlier calls (other column blocks)
    int64_t col0;      // index of column 0 in the keys
    const float *M;    // [m, ldm] smallest value of every chunk of 32 columns, or null (every column is read)
    int64_t ldm;
    float *tau_out;    // [m] or null (requires S == 1): the value of the row's k-th entry afterwards, +inf if short of k
};

hipError_t launch_valu_calibration(int64_t pairs_per_wave, int blocks, float *sink, hipStream_t stream);
hipError_t launch_mfma_calibration(int64_t mfma_per_wave, int blocks, float *sink, hipStream_t stream);
hipError_t launch_contraction_calibration(int shape, int dc, int64_t tiles, int blocks, const float *rows, float *sink,
                                          hipStream_t stream);   // shape 0 / 1, dc 16 / 32 / 64; rows: [64, 256] floats
hipError_t launch_mfma_bf16_calibration(int64_t mfma_per_wave, int blocks, int chains, float *sink, hipStream_t stream);   // chains: 4 or 2
hipError_t launch_read_calibration(const float *buf, int64_t n_floats, int64_t floats_per_wave, float *sink,
                                   hipStream_t stream);   // sizes: multiples of 2048 floats
hipError_t launch_fold(const FoldArgs &a, hipStream_t stream);
hipError_t launch_fold_dist(const FoldDistArgs &a, int mode, hipStream_t stream);
hipError_t launch_pack(const PackArgs &a, hipStream_t stream);
hipError_t launch_select(const SelectArgs &a, hipStream_t stream);
hipError_t launch_prep(const PrepArgs &a, hipStream_t stream);
hipError_t launch_col_mean(const float *X, int64_t n, int32_t d, int32_t dpad, double *sums, float *mu, hipStream_t stream);   // mu[dpad] = column means, 0 beyond d
hipError_t launch_prep_split(const SplitPrepArgs &a, hipStream_t stream);
hipError_t launch_tiles_split(const TileArgs &a, int waves, hipStream_t stream);   // dpad: multiple of 32, <= 256; waves = 8; n_qtiles in tiles of 32 * waves queries
hipError_t launch_zero_word(int32_t *word, hipStream_t stream);
hipError_t launch_gather_rows(const GatherArgs &a, hipStream_t stream);
hipError_t launch_tiles_qreg_subset(const TileArgs &a, hipStream_t stream);   // nq = capacity of the subset; S > 1 needs bound
hipError_t launch_tiles(const TileArgs &a, hipStream_t stream);
hipError_t launch_tiles_qreg(const TileArgs &a, hipStream_t stream);   // dpad: multiple of 32, <= 256
hipError_t launch_dist_qreg(const DistArgs &a, int n_qtiles, int mode, hipStream_t stream);      // mode: see DIST_*
hipError_t launch_dist_stream(const DistArgs &a, int n_qtiles, int mode, hipStream_t stream);    // any dpad (multiple of KNN_DC); n_rt, chunk in tiles of 128 rows   // dpad: multiple of 32, <= 256
hipError_t launch_finalize(const FinArgs &a, hipStream_t stream);
hipError_t launch_reduce_max(const float *c, int64_t n, float *out, hipStream_t stream);
hipError_t launch_pairs_qreg(const PairArgs &a, int blocks, bool split, hipStream_t stream);   // split: operands are bf16 pieces (prep_split)

}  // namespace knn
#endif
