/*
 * knn.h -- C ABI of the MI355X (gfx950) exact k-nearest-neighbour library.
 *
 * The library solves the problem stated in Sect. 3 of Kato & Hosino, "Solving
 * k-Nearest Neighbor Problem on Multiple Graphics Processors": for every query
 * vector, the k reference vectors at the smallest distance, listed in
 * non-decreasing order of distance, every reference left out being at least as
 * far as the k-th one listed.  It does so by brute force, as the paper does
 * (Sect. 4-6): a tiled all-pairs distance computation and a per-row selection
 * of the k smallest.  Two organisations exist (knn_plan_t): FUSED, one pass in
 * which the selection runs on the distance tile while it is still in registers
 * and no distance is ever stored; and TWO-PHASE, the paper's own organisation,
 * which keeps distances in the caller's workspace between the two phases.  The
 * library takes the faster one that fits the workspace it is given.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; the library
 *     allocates and frees nothing and keeps no pointer after it returns.
 *   - Matrices are row-major, contiguous, fp32; row stride == d.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it and the call returns without waiting; results are
 *     valid once the caller has synchronised the stream.  (Exception: a call
 *     given a profile record waits for its own work, see knn_options_t.)
 *   - Errors are return codes; nothing aborts or throws.  On any error other
 *     than KNN_EDEVICE nothing has been enqueued.
 *   - Indices are 0-based reference row numbers (the paper counts from 1).
 *   - Ties in distance go to the lower reference index (the paper allows any
 *     resolution).  A query is never its own neighbour when it is declared to
 *     be a member of the reference set (Sect. 4: only pairs x > y are computed);
 *     exclusion is by row number, so another row with equal coordinates is an
 *     ordinary neighbour at distance 0.
 *   - Which k references win is decided on single-precision values of the
 *     expanded form (|r|^2 - 2 q.r for the squared Euclidean distance), whose
 *     absolute error is a few 2^-24 (|q|^2 + |r|^2).  References whose true
 *     distances to a query differ by less than that may be ranked either way;
 *     for data far from the origin (all rows sharing a large offset) that band
 *     is wide relative to the distances themselves: centre such data first
 *     (subtracting one vector from every row changes no distance), or set
 *     knn_options_t.center, which does so inside the call.  The distances
 *     REPORTED are recomputed from the original rows in double.
 *   - NaN or infinite input values: behaviour undefined.
 */
#ifndef KNN_H_
#define KNN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KNN_SQEUCLIDEAN = 0, /* sum_c (u_c - v_c)^2 */
    KNN_COSINE = 1,      /* 1 - u.v / (|u| |v|); 1 if either vector is all zero */
    KNN_HELLINGER = 2,   /* sum_c (sqrt u_c - sqrt v_c)^2, the distance of the paper's experiment
                            (Sect. 7, Eq. 1, with the square its printed form lacks);
                            inputs must be >= 0 */
    /* Sect. 3 asks of a distance only that it be a fold over the coordinates,
       a_{c+1} = dbar(u_c, v_c, a_c).  The three above reduce to an inner product and run on
       the matrix cores; so does KNN_KL.  KNN_L1 and KNN_LINF do not: they run the fold
       itself on the vector ALUs (a separate kernel, bound by the vector instruction rate). */
    KNN_L1 = 3,          /* sum_c |u_c - v_c| */
    KNN_LINF = 4,        /* max_c |u_c - v_c| */
    KNN_KL = 5           /* sum_c q_c ln(q_c / r_c), the QUERY first; terms with q_c = 0 count 0.
                            Not symmetric (Sect. 3 notes that such a distance needs both orders
                            of every pair): knn_build evaluates the full square for it.
                            Inputs must be >= 0, references > 0 wherever a query is > 0; no
                            normalisation is applied or required */
} knn_metric_t;

typedef enum {
    KNN_OK = 0,
    KNN_EINVAL = 1,       /* null pointer, size or option out of range, k too large for the set */
    KNN_EUNSUPPORTED = 2, /* k above KNN_MAX_K, nr >= 2^31, or a plan that cannot serve the call */
    KNN_ENOMEM = 3,       /* workspace smaller than the smallest plan needs */
    KNN_EDEVICE = 4       /* a HIP call failed (no gfx950 device, launch error) */
} knn_status_t;

#define KNN_MAX_K 128

/* How the two stages of the method (Sect. 5: distances, Sect. 6: k smallest per row) are run. */
typedef enum {
    KNN_PLAN_AUTO = 0,            /* the fastest plan whose workspace fits the one passed */
    KNN_PLAN_FUSED_STREAMING = 1, /* fused; both operands staged through LDS; any d */
    KNN_PLAN_FUSED = 3,           /* fused; query operands resident in registers (d <= 256,
                                     else as 1).  Workspace about 4 n d + 8 n kcap bytes */
    KNN_PLAN_TWO_PHASE = 4,       /* distances written to the workspace, then selected from:
                                     the whole matrix, or (knn_build, symmetric distance) two
                                     blocks of block_rows^2 at a time, walked by pairs of row
                                     panels; chunks of distances that can no longer enter a
                                     row's list are then not stored */
    KNN_PLAN_SPLIT_BF16 = 6       /* experiment, never taken by AUTO: fused; operands split into two
                                     bf16 pieces, three bf16 matrix products per pair pick K' > k
                                     candidates per query, which are then priced exactly; rows the
                                     error bound of the split cannot prove right are answered
                                     again by the fp32 kernel (at most 4096 rows).  Full square
                                     unless knn_build is asked for symmetric = 1.
                                     KNN_SQEUCLIDEAN, d <= 256 and k <= 112 only */
} knn_plan_t;

/* Time spent by one call, filled in when knn_options_t.profile points here. */
typedef struct {
    float ms_prepare;   /* row norms / scaled copies            (Sect. 5 prologue) */
    float ms_main;      /* distance + selection kernel(s)       (Sect. 5 and 6)    */
    float ms_finalize;  /* merge of partial lists, re-score, final order            */
    float ms_total;
    int32_t main_launches; /* kernel launches counted in ms_main */
    int32_t symmetric;     /* 1 if each unordered pair of rows was evaluated once */
    int64_t pairs_computed;/* (query, reference) pairs whose distance was evaluated,
                              padding of ragged tiles included */
    float ms_select;       /* two-phase plans: the part of ms_main not spent in the distance kernel */
    int32_t two_phase;     /* 0: fused.  1: whole matrix.  2: by pairs of row panels */
} knn_profile_t;

/* Optional knobs; pass NULL for defaults.  Zero-initialise, then set fields. */
typedef struct {
    int32_t symmetric;  /* knn_build only: 0 = auto, 1 = evaluate each unordered pair of rows once
                           (Sect. 3-4; fused: a tournament of block pairs), 2 = the full square */
    int32_t rescore;    /* 0 / 1 = report distances recomputed from the original rows with double
                           accumulation; 2 = report the single-precision values selected on */
    int32_t r_splits;   /* 0 = auto.  Fused plans: slices of the reference range per query tile,
                           each with a partial list per query, merged at the end */
    int32_t variant;    /* a knn_plan_t; KNN_PLAN_AUTO never fails for lack of workspace as long as
                           the fused plan fits */
    int32_t block_rows; /* 0 = auto.  Fused symmetric schedule: rows per block (multiple of 128).
                           KNN_PLAN_TWO_PHASE with knn_build: rows per panel (multiple of 256),
                           and the panel walk is used whatever the size */
    int32_t center;     /* 0 = off.  1 = KNN_SQEUCLIDEAN: subtract the references' column means (summed
                           in double, once per call) from every query and reference row before
                           the expanded form is taken -- no squared Euclidean distance changes,
                           and the error of the expanded form (see the conventions above) then scales with
                           the spread of the data, not with its distance from the origin.  Costs
                           one more pass over R, a copy of R where the plan had none, and
                           12 * dpad bytes of workspace.  Ignored for the other distances */
    knn_profile_t *profile; /* HOST pointer or NULL.  If set, the call brackets its kernels with
                           events, waits for them and fills this in */
    int32_t *uncertified;   /* DEVICE pointer or NULL; KNN_PLAN_SPLIT_BF16 only: receives the number
                           of query rows whose answer is neither proven exact by the error bound of
                           the split products nor recomputed by the fp32 kernel, i.e. those beyond
                           the 4096 the second pass takes (such rows are still answered, from the
                           candidates kept) */
} knn_options_t;

/* What a call with these sizes, options and workspace size would do; see knn_plan(). */
typedef struct {
    int32_t plan;           /* the knn_plan_t taken */
    int32_t symmetric;      /* 1: each unordered pair of rows evaluated once */
    int32_t two_phase;      /* as knn_profile_t.two_phase */
    int32_t main_launches;  /* kernel launches of the distance + selection stage */
    uint64_t workspace_bytes; /* what this plan needs */
    char kernel[32];        /* name of the kernel that does the distance arithmetic */
} knn_plan_info_t;

/*
 * All-pairs self kNN (Sect. 3): neighbours of every row of X among the other
 * rows of X.
 *   X    [n, d]  device, read only
 *   idx  [n, k]  device, int32, out
 *   dist [n, k]  device, fp32, out, ascending per row
 *   workspace    device, 256-byte aligned, uninitialised; garbage afterwards.
 *                With default options: the plan is the fastest one that fits
 *                workspace_bytes.  knn_workspace_bytes() is what the preferred plan
 *                wants (it may hold distances: up to 72 GiB, 37 GB at n = 2^20),
 *                knn_workspace_bytes_min() what the fused plan needs; anything in
 *                between works, less is KNN_ENOMEM.
 * Requires 2 <= n < 2^31, 1 <= d, 1 <= k <= min(n-1, KNN_MAX_K).
 */
knn_status_t knn_build(const float *X, int64_t n, int32_t d, int32_t k, knn_metric_t metric,
                       int32_t *idx, float *dist,
                       void *workspace, size_t workspace_bytes, void *stream);

knn_status_t knn_build_ex(const float *X, int64_t n, int32_t d, int32_t k, knn_metric_t metric,
                          int32_t *idx, float *dist,
                          void *workspace, size_t workspace_bytes, void *stream,
                          const knn_options_t *opt);

/*
 * Query / reference form, the two-set shape of the paper's distance procedure
 * (Sect. 5, CalcDistances(d, n1, {v1}, n2, {v2})) and the unit of blocking:
 * neighbours of every row of Q among the rows of R.
 *   Q [nq, d], R [nr, d]  device, read only (may alias)
 *   self_offset >= 0: query i IS reference row self_offset + i and that pair is
 *                     skipped (requires self_offset + nq <= nr); -1: no such relation.
 *   idx [nq, k], dist [nq, k]  device, out
 *   workspace: as for knn_build.
 * Requires 1 <= nq, 1 <= nr < 2^31, 1 <= k <= min(nr - (self_offset >= 0), KNN_MAX_K).
 */
knn_status_t knn_search(const float *Q, int64_t nq, const float *R, int64_t nr, int32_t d,
                        int32_t k, knn_metric_t metric, int64_t self_offset,
                        int32_t *idx, float *dist,
                        void *workspace, size_t workspace_bytes, void *stream);

knn_status_t knn_search_ex(const float *Q, int64_t nq, const float *R, int64_t nr, int32_t d,
                           int32_t k, knn_metric_t metric, int64_t self_offset,
                           int32_t *idx, float *dist,
                           void *workspace, size_t workspace_bytes, void *stream,
                           const knn_options_t *opt);

/*
 * knn_search for callers that cannot allocate device memory and have no workspace to
 * bring: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments and results as knn_search with default options, but the
 * workspace is a static device array of KNN_STATIC_SCRATCH_BYTES inside the library
 * (one per GPU, held until the process ends); the call itself allocates nothing.
 * Sizes whose smallest plan needs more than that are refused with KNN_ENOMEM and
 * nothing is enqueued (roughly: 4 d (nq + nr) + 8 kcap S nq bytes must fit, kcap = k
 * rounded up to 16/32/64/128, S the number of reference slices, 16 for small nq).
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU
 * (different streams or threads) race; calls on one stream are safe back to back.
 */
#define KNN_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
knn_status_t knn_search_static(const float *Q, int64_t nq, const float *R, int64_t nr, int32_t d,
                               int32_t k, knn_metric_t metric, int64_t self_offset,
                               int32_t *idx, float *dist, void *stream);

/*
 * Bytes of device workspace the PREFERRED plan of a call with these sizes and default
 * options wants; 0 if the sizes are invalid.  `symmetric` != 0 asks for knn_build (nq is
 * ignored, nr = n), 0 for knn_search.
 */
size_t knn_workspace_bytes(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric,
                           int32_t symmetric);

/* Same, for a given option block; 0 also if an option is out of range. */
size_t knn_workspace_bytes_ex(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric,
                              int32_t symmetric, const knn_options_t *opt);

/* The smallest workspace with which a call with default options succeeds (the fused plan's:
   scaled copies of the inputs and the lists). */
size_t knn_workspace_bytes_min(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric,
                               int32_t symmetric);

/*
 * The plan a call with these sizes and options would take if given a workspace of
 * `workspace_bytes` (SIZE_MAX: no limit), without running anything: `out` is a HOST
 * pointer.  KNN_ENOMEM if no plan fits, otherwise the status the call itself would
 * return for these sizes and options.
 */
knn_status_t knn_plan(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric,
                      int32_t symmetric, const knn_options_t *opt, size_t workspace_bytes,
                      knn_plan_info_t *out);

/*
 * Batched partial sort of a matrix that already exists in memory: the paper's Phase 2 as
 * a routine of its own (Sect. 6, KSmallest(k, n, m, {h_i}, {a_ij}); Sect. 8 singles it out
 * as useful beyond kNN).  For every row of A, the k smallest entries in non-decreasing
 * order and their column numbers; equal values go to the lower column.
 *   A   [m, lda] device, fp32, row stride lda >= n floats, read only (read exactly once)
 *   idx [m, k]   device, int32, out: column numbers
 *   val [m, k]   device, fp32, out: the values, bit-identical copies of entries of A
 * Requires 1 <= m < 2^31, 1 <= k <= min(n, KNN_MAX_K), n < 2^31.  Rows whose start is
 * 16-byte aligned (A aligned, lda % 4 == 0) are read with 128-bit loads.
 */
knn_status_t knn_select(const float *A, int64_t m, int64_t n, int64_t lda, int32_t k,
                        int32_t *idx, float *val,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of device workspace knn_select needs (256-byte aligned); 0 if the sizes are invalid. */
size_t knn_select_workspace_bytes(int64_t m, int64_t n, int32_t k);

/*
 * Calibration, not part of the method: launches a kernel that does nothing but issue
 * v_mfma_f32_32x32x2_f32 (the instruction of the fused kernels' contraction) from
 * `waves_per_simd` (1..4) waves on every SIMD of the device, `mfma_per_wave` of them per wave
 * on four independent accumulators, so that a caller who times the launch learns the matrix
 * rate this device sustains under load, to put beside the nominal peak.  One launch executes
 * waves * mfma_per_wave * 4096 flop, waves = *total_waves (HOST pointer, may be NULL).
 *   sink  device buffer of at least 4 * 64 * 4 * (compute units) * waves_per_simd bytes
 *         (one float per lane; the value is meaningless, it keeps the work observable)
 * Asynchronous on `stream`.  KNN_EINVAL for bad arguments, KNN_EDEVICE on a launch error.
 */
knn_status_t knn_mfma_calibration(int64_t mfma_per_wave, int32_t waves_per_simd, float *sink,
                                  size_t sink_bytes, int64_t *total_waves, void *stream);

/*
 * The same for v_mfma_f32_32x32x16_bf16, the instruction of KNN_PLAN_SPLIT_BF16: one launch
 * executes waves * mfma_per_wave * 32768 flop.  `chains` is the number of independent
 * accumulators per wave the instructions rotate over: 4, or 2 (the dependency pattern of that
 * plan's kernel).  Other arguments and errors as for knn_mfma_calibration.
 */
knn_status_t knn_mfma_bf16_calibration(int64_t mfma_per_wave, int32_t waves_per_simd, int32_t chains,
                                       float *sink, size_t sink_bytes, int64_t *total_waves, void *stream);

/*
 * Calibration of two design choices of the fp32 tile kernels: their contraction and nothing
 * else -- a workgroup of 4 waves, 32 queries per wave resident in registers (d = 256), 64
 * reference rows staged through swizzled LDS `dc` coordinates per step (16, 32 or 64; the
 * kernels use 32), no selection -- on v_mfma_f32_32x32x2_f32 (`shape` 0, the kernels' choice) or
 * v_mfma_f32_16x16x4_f32 (`shape` 1).  Two workgroups per compute unit, each contracting
 * `tiles_per_workgroup` tiles of 128 queries x 64 references x 256 coordinates (4 194 304 flop).
 *   rows   DEVICE, 16-byte aligned, [64, 256] fp32: the reference rows every tile re-reads
 *   sink   DEVICE, at least 4 * 256 * 2 * (compute units) bytes
 *   workgroups  HOST pointer or NULL: receives the number launched
 * Asynchronous on `stream`.  Errors as for knn_mfma_calibration.
 */
knn_status_t knn_contraction_calibration(int32_t shape, int32_t dc, int64_t tiles_per_workgroup,
                                         const float *rows, float *sink, size_t sink_bytes,
                                         int64_t *workgroups, void *stream);

/*
 * The same for the vector ALUs: every wave issues `pairs_per_wave` times the fold kernel's
 * instruction pair (v_sub_f32 with a scalar operand, v_add_f32 with the |.| modifier) on 32
 * independent accumulators.  One launch executes waves * pairs_per_wave * 2 * 64 lane
 * operations.  pairs_per_wave must be a positive multiple of 128, waves_per_simd 1..8, and
 * the sink 64 bytes larger than knn_mfma_calibration asks for (the kernel's 16 operand values
 * are copied there from the host, asynchronously, before the launch).  Errors as for
 * knn_mfma_calibration.
 */
knn_status_t knn_valu_calibration(int64_t pairs_per_wave, int32_t waves_per_simd, float *sink,
                                  size_t sink_bytes, int64_t *total_waves, void *stream);

/*
 * The same for the memory: reads `n_floats` floats from `buf` (DEVICE pointer, 16-byte aligned)
 * exactly once, the way the selection kernel of knn_select reads the rows of its matrix -- every
 * wave a contiguous range of `floats_per_wave`, eight 16-byte loads in flight per lane -- and
 * does nothing with them but keep a minimum.  A caller who times the launch learns the read
 * rate the device's memory sustains (4 * n_floats bytes per launch), to put beside the nominal
 * HBM peak and beside knn_select's own rate.  Both counts must be positive multiples of 2048;
 * the sink (DEVICE pointer) must hold 1024 floats.  Errors as for knn_mfma_calibration.
 */
knn_status_t knn_read_calibration(const float *buf, int64_t n_floats, int64_t floats_per_wave, float *sink,
                                  size_t sink_bytes, void *stream);

/* Static, human-readable name of a status code. */
const char *knn_status_string(knn_status_t status);

/* Text of the last HIP error seen by this thread's calls ("" if none). */
const char *knn_last_device_error(void);

#ifdef __cplusplus
}
#endif
#endif /* KNN_H_ */
