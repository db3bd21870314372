// Device code of the exact kNN library for MI355X (gfx950, wave64): one translation unit.
//
//   knn_select_common.h  packed keys, rank merges, the selection's rare path
//   knn_rows_kernels.h   prep_rows, select_rows, finalize_rows, reduce_max      (HBM bound)
//   knn_tiles_kernels.h  the fused kernels of the full-square schedule: distance tiles on the
//                        fp32 matrix cores, threshold test and k-best update in the epilogue;
//                        the distance matrix of the paper's Phase 1 (Sect. 5) is never written
//                        out, its Phase 2 (Sect. 6) runs on the accumulators
//   knn_pairs_kernel.h   the symmetric schedule (Sect. 3-4)
//   knn_matrix_kernel.h  Phase 1 on its own: the distance matrix written out (Sect. 5), for the
//                        problems where selecting from it afterwards (select_rows) is cheaper
//   knn_fold_kernels.h   folds that are not inner products, on the vector ALUs; calibration
//   knn_split_kernels.h  experiment: the fused kernel on bf16 matrix instructions, operands
//                        split into two pieces, used as a filter with a proven error bound
//   knn_calibration_kernels.h  the fp32 contraction alone, by matrix instruction and LDS step width
//   this file            launchers called from the C ABI (knn_api.cpp)
//
// On the matrix path distances are evaluated in the expanded form
//   p(q, j) = c_j + sum_c Q'[q][c] R'[j][c]:
//   squared Euclidean:  Q' = -2 Q, R' = R,      c_j = |r_j|^2;  delta = p + |q|^2
//   cosine:             Q' = -Q/|Q|, R' = R/|R|, c_j = 0;        delta = p + 1
//   Hellinger:          the squared Euclidean form on sqrt(x);  Kullback-Leibler: Q' = -q,
//                       R' = ln r, c_j = 0; delta = p + sum q ln q
// which is the paper's coordinate-wise fold (Sect. 3, "cumulatively computable")
// with a multiply-add as the step, so the d-loop is a matrix product.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "knn_device.h"

namespace knn {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));   // one operand of v_mfma_f32_32x32x16_bf16
typedef __attribute__((address_space(3))) void *lds_ptr;

}  // namespace knn

#include "knn_select_common.h"
#include "knn_rows_kernels.h"
#include "knn_tiles_kernels.h"
#include "knn_pairs_kernel.h"
#include "knn_matrix_kernel.h"
#include "knn_fold_kernels.h"
#include "knn_split_kernels.h"
#include "knn_calibration_kernels.h"

namespace knn {

hipError_t launch_valu_calibration(int64_t pairs_per_wave, int blocks, float *sink, hipStream_t stream)
{
    // the seed values live at the end of the sink, past the part the kernel writes
    const float *seed = sink + (int64_t)blocks * 256;
    hipLaunchKernelGGL(valu_only, dim3((unsigned)blocks), dim3(256), 0, stream, pairs_per_wave / 128, seed, sink);
    return hipGetLastError();
}

hipError_t launch_read_calibration(const float *buf, int64_t n_floats, int64_t floats_per_wave, float *sink,
                                   hipStream_t stream)
{
    const int64_t n_pieces = n_floats / SEL_CHUNK, ppw = floats_per_wave / SEL_CHUNK;
    const int64_t waves = (n_pieces + ppw - 1) / ppw;
    hipLaunchKernelGGL(read_only, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, stream, buf, n_pieces, ppw, sink);
    return hipGetLastError();
}

hipError_t launch_mfma_calibration(int64_t mfma_per_wave, int blocks, float *sink, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_only, dim3((unsigned)blocks), dim3(256), 0, stream, mfma_per_wave / 16, sink);
    return hipGetLastError();
}

hipError_t launch_contraction_calibration(int shape, int dc, int64_t tiles, int blocks, const float *rows, float *sink,
                                          hipStream_t stream)
{
    dim3 grid((unsigned)blocks), block(256);
#define KNN_CONTRACT_CASE(S, C)                                                                      \
    if (shape == S && dc == C) {                                                                     \
        hipLaunchKernelGGL((contract_only<S, C>), grid, block, 0, stream, rows, tiles, sink);        \
        return hipGetLastError();                                                                    \
    }
    KNN_CONTRACT_CASE(0, 16)
    KNN_CONTRACT_CASE(0, 32)
    KNN_CONTRACT_CASE(0, 64)
    KNN_CONTRACT_CASE(1, 16)
    KNN_CONTRACT_CASE(1, 32)
    KNN_CONTRACT_CASE(1, 64)
#undef KNN_CONTRACT_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_mfma_bf16_calibration(int64_t mfma_per_wave, int blocks, int chains, float *sink, hipStream_t stream)
{
    if (chains == 4)
        hipLaunchKernelGGL(mfma_bf16_only<4>, dim3((unsigned)blocks), dim3(256), 0, stream, mfma_per_wave / 16, sink);
    else if (chains == 2)
        hipLaunchKernelGGL(mfma_bf16_only<2>, dim3((unsigned)blocks), dim3(256), 0, stream, mfma_per_wave / 16, sink);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}


// ---------------------------------------------------------------------------
// launchers (called from the C ABI in knn_api.cpp)
// ---------------------------------------------------------------------------
hipError_t launch_prep(const PrepArgs &a, hipStream_t stream)
{
    int64_t blocks = (a.n + 3) / 4;
    int64_t pad_blocks = (a.n_cpad - a.n + 255) / 256;
    if (blocks > 262144) blocks = 262144;
    if (blocks < pad_blocks) blocks = pad_blocks;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(prep_rows, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_col_mean(const float *X, int64_t n, int32_t d, int32_t dpad, double *sums, float *mu, hipStream_t stream)
{
    const unsigned cb = (unsigned)((dpad + 255) / 256);
    int64_t ry = (n + 63) / 64;                    // at least 64 rows per thread
    if (ry > 1024) ry = 1024;
    if (ry < 1) ry = 1;
    hipLaunchKernelGGL(col_zero, dim3(cb), dim3(256), 0, stream, sums, dpad);
    hipLaunchKernelGGL(col_sum, dim3((unsigned)((d + 255) / 256), (unsigned)ry), dim3(256), 0, stream, X, n, d, sums);
    hipLaunchKernelGGL(col_mean, dim3(cb), dim3(256), 0, stream, sums, n, d, dpad, mu);
    return hipGetLastError();
}

hipError_t launch_tiles(const TileArgs &a, hipStream_t stream)
{
    int64_t blocks = (int64_t)a.n_qtiles * a.S;
    hipLaunchKernelGGL(knn_tiles, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

template <bool SHARE>
static hipError_t launch_tiles_qreg_t(const TileArgs &a, hipStream_t stream)
{
    int64_t blocks = (int64_t)a.n_qtiles * a.S;
    dim3 grid((unsigned)blocks), block(256);
    switch (a.dpad) {
    case 32: hipLaunchKernelGGL((knn_tiles_qreg<32, SHARE>), grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL((knn_tiles_qreg<64, SHARE>), grid, block, 0, stream, a); break;
    case 96: hipLaunchKernelGGL((knn_tiles_qreg<96, SHARE>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((knn_tiles_qreg<128, SHARE>), grid, block, 0, stream, a); break;
    case 160: hipLaunchKernelGGL((knn_tiles_qreg<160, SHARE>), grid, block, 0, stream, a); break;
    case 192: hipLaunchKernelGGL((knn_tiles_qreg<192, SHARE>), grid, block, 0, stream, a); break;
    case 224: hipLaunchKernelGGL((knn_tiles_qreg<224, SHARE>), grid, block, 0, stream, a); break;
    case 256: hipLaunchKernelGGL((knn_tiles_qreg<256, SHARE>), grid, block, 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_tiles_qreg(const TileArgs &a, hipStream_t stream)
{
    // slices share their bound only when there is more than one of them
    return a.bound != nullptr && a.S > 1 ? launch_tiles_qreg_t<true>(a, stream) : launch_tiles_qreg_t<false>(a, stream);
}

template <int MODE>
static hipError_t launch_dist_qreg_t(const DistArgs &a, int n_qtiles, hipStream_t stream)
{
    dim3 grid((unsigned)((int64_t)n_qtiles * a.n_chunks)), block(256);
    switch (a.dpad) {
    case 32: hipLaunchKernelGGL((knn_dist_qreg<32, MODE>), grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL((knn_dist_qreg<64, MODE>), grid, block, 0, stream, a); break;
    case 96: hipLaunchKernelGGL((knn_dist_qreg<96, MODE>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((knn_dist_qreg<128, MODE>), grid, block, 0, stream, a); break;
    case 160: hipLaunchKernelGGL((knn_dist_qreg<160, MODE>), grid, block, 0, stream, a); break;
    case 192: hipLaunchKernelGGL((knn_dist_qreg<192, MODE>), grid, block, 0, stream, a); break;
    case 224: hipLaunchKernelGGL((knn_dist_qreg<224, MODE>), grid, block, 0, stream, a); break;
    case 256: hipLaunchKernelGGL((knn_dist_qreg<256, MODE>), grid, block, 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_dist_stream(const DistArgs &a, int n_qtiles, int mode, hipStream_t stream)
{
    dim3 grid((unsigned)((int64_t)n_qtiles * a.n_chunks)), block(256);
    switch (mode) {
    case DIST_FULL: hipLaunchKernelGGL(knn_dist_stream<DIST_FULL>, grid, block, 0, stream, a); break;
    case DIST_TRIANGLE: hipLaunchKernelGGL(knn_dist_stream<DIST_TRIANGLE>, grid, block, 0, stream, a); break;
    case DIST_RECT_MIRROR: hipLaunchKernelGGL(knn_dist_stream<DIST_RECT_MIRROR>, grid, block, 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_dist_qreg(const DistArgs &a, int n_qtiles, int mode, hipStream_t stream)
{
    switch (mode) {
    case DIST_FULL: return launch_dist_qreg_t<DIST_FULL>(a, n_qtiles, stream);
    case DIST_TRIANGLE: return launch_dist_qreg_t<DIST_TRIANGLE>(a, n_qtiles, stream);
    case DIST_RECT_MIRROR: return launch_dist_qreg_t<DIST_RECT_MIRROR>(a, n_qtiles, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_reduce_max(const float *c, int64_t n, float *out, hipStream_t stream)
{
    hipLaunchKernelGGL(reduce_max, dim3(1), dim3(1024), 0, stream, c, n, out);
    return hipGetLastError();
}

template <bool SPLIT>
static hipError_t launch_pairs_qreg_t(const PairArgs &a, int blocks, hipStream_t stream)
{
    dim3 grid((unsigned)blocks), block(256);
    switch (a.dpad) {
    case 32: hipLaunchKernelGGL((knn_pairs_qreg<32, true, SPLIT>), grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL((knn_pairs_qreg<64, true, SPLIT>), grid, block, 0, stream, a); break;
    case 96: hipLaunchKernelGGL((knn_pairs_qreg<96, true, SPLIT>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((knn_pairs_qreg<128, true, SPLIT>), grid, block, 0, stream, a); break;
    case 160: hipLaunchKernelGGL((knn_pairs_qreg<160, true, SPLIT>), grid, block, 0, stream, a); break;
    case 192: hipLaunchKernelGGL((knn_pairs_qreg<192, true, SPLIT>), grid, block, 0, stream, a); break;
    case 224: hipLaunchKernelGGL((knn_pairs_qreg<224, true, SPLIT>), grid, block, 0, stream, a); break;
    case 256:
        // at the register limit: the mask scan costs the matrix loop spills that only pay
        // while candidates are frequent, i.e. for the smaller problems
        if (a.n < (1 << 19))
            hipLaunchKernelGGL((knn_pairs_qreg<256, true, SPLIT>), grid, block, 0, stream, a);
        else
            hipLaunchKernelGGL((knn_pairs_qreg<256, false, SPLIT>), grid, block, 0, stream, a);
        break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_pairs_qreg(const PairArgs &a, int blocks, bool split, hipStream_t stream)
{
    return split ? launch_pairs_qreg_t<true>(a, blocks, stream) : launch_pairs_qreg_t<false>(a, blocks, stream);
}

hipError_t launch_fold(const FoldArgs &a, hipStream_t stream)
{
    const int64_t groups = (a.nq + 63) / 64;
    const int64_t blocks = ((groups + FOLD_WAVES - 1) / FOLD_WAVES * a.S + 7) / 8 * 8;
    if (a.metric == 3)
        hipLaunchKernelGGL(knn_fold<3>, dim3((unsigned)blocks), dim3(64 * FOLD_WAVES), 0, stream, a);
    else if (a.metric == 4)
        hipLaunchKernelGGL(knn_fold<4>, dim3((unsigned)blocks), dim3(64 * FOLD_WAVES), 0, stream, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

template <int METRIC>
static hipError_t launch_fold_dist_t(const FoldDistArgs &a, int mode, hipStream_t stream)
{
    dim3 grid((unsigned)((int64_t)a.n_qblocks * a.n_chunks)), block(64 * FOLD_WAVES);
    switch (mode) {
    case DIST_FULL: hipLaunchKernelGGL((knn_fold_dist<METRIC, DIST_FULL>), grid, block, 0, stream, a); break;
    case DIST_TRIANGLE: hipLaunchKernelGGL((knn_fold_dist<METRIC, DIST_TRIANGLE>), grid, block, 0, stream, a); break;
    case DIST_RECT_MIRROR: hipLaunchKernelGGL((knn_fold_dist<METRIC, DIST_RECT_MIRROR>), grid, block, 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_fold_dist(const FoldDistArgs &a, int mode, hipStream_t stream)
{
    if (a.metric == 3) return launch_fold_dist_t<3>(a, mode, stream);
    if (a.metric == 4) return launch_fold_dist_t<4>(a, mode, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_pack(const PackArgs &a, hipStream_t stream)
{
    int64_t total = (a.n + a.rows_per_tile - 1) / a.rows_per_tile * a.rows_per_tile * (int64_t)(a.dpad >> 2);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(pack_tiles, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_select(const SelectArgs &a, hipStream_t stream)
{
    int64_t blocks = (a.m * a.S + 3) / 4;
    if (a.M != nullptr)
        hipLaunchKernelGGL(select_rows_sparse, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL(select_rows, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_prep_split(const SplitPrepArgs &a, hipStream_t stream)
{
    int64_t blocks = (a.n + 3) / 4;
    int64_t pad_blocks = a.c_out ? (a.n_cpad - a.n + 255) / 256 : 0;
    if (blocks > 262144) blocks = 262144;
    if (blocks < pad_blocks) blocks = pad_blocks;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(prep_split, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

template <int WAVES, bool SHARE>
static hipError_t launch_tiles_split_t(const TileArgs &a, hipStream_t stream)
{
    int64_t blocks = (int64_t)a.n_qtiles * a.S;
    dim3 grid((unsigned)blocks), block(64 * WAVES);
    switch (a.dpad) {
    case 32: hipLaunchKernelGGL((knn_tiles_split<32, WAVES, SHARE>), grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL((knn_tiles_split<64, WAVES, SHARE>), grid, block, 0, stream, a); break;
    case 96: hipLaunchKernelGGL((knn_tiles_split<96, WAVES, SHARE>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((knn_tiles_split<128, WAVES, SHARE>), grid, block, 0, stream, a); break;
    case 160: hipLaunchKernelGGL((knn_tiles_split<160, WAVES, SHARE>), grid, block, 0, stream, a); break;
    case 192: hipLaunchKernelGGL((knn_tiles_split<192, WAVES, SHARE>), grid, block, 0, stream, a); break;
    case 224: hipLaunchKernelGGL((knn_tiles_split<224, WAVES, SHARE>), grid, block, 0, stream, a); break;
    case 256: hipLaunchKernelGGL((knn_tiles_split<256, WAVES, SHARE>), grid, block, 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_tiles_split(const TileArgs &a, int waves, hipStream_t stream)
{
    const bool share = a.bound != nullptr && a.S > 1;
    if (waves != 8) return hipErrorInvalidValue;
    return share ? launch_tiles_split_t<8, true>(a, stream) : launch_tiles_split_t<8, false>(a, stream);
}

hipError_t launch_gather_rows(const GatherArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(gather_rows, dim3((unsigned)((a.cap + 3) / 4)), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_tiles_qreg_subset(const TileArgs &a, hipStream_t stream)
{
    if (a.nq_dev == nullptr || a.self_rows == nullptr || (a.S > 1 && a.bound == nullptr)) return hipErrorInvalidValue;
    int64_t blocks = (int64_t)a.n_qtiles * a.S;
    dim3 grid((unsigned)blocks), block(256);
    switch (a.dpad) {
    case 32: hipLaunchKernelGGL((knn_tiles_qreg<32, true, true>), grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL((knn_tiles_qreg<64, true, true>), grid, block, 0, stream, a); break;
    case 96: hipLaunchKernelGGL((knn_tiles_qreg<96, true, true>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((knn_tiles_qreg<128, true, true>), grid, block, 0, stream, a); break;
    case 160: hipLaunchKernelGGL((knn_tiles_qreg<160, true, true>), grid, block, 0, stream, a); break;
    case 192: hipLaunchKernelGGL((knn_tiles_qreg<192, true, true>), grid, block, 0, stream, a); break;
    case 224: hipLaunchKernelGGL((knn_tiles_qreg<224, true, true>), grid, block, 0, stream, a); break;
    case 256: hipLaunchKernelGGL((knn_tiles_qreg<256, true, true>), grid, block, 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

__global__ void zero_word(int32_t *w) { *w = 0; }

// a one-thread fill kernel rather than hipMemsetAsync, so that a caller may capture the call in a graph
hipError_t launch_zero_word(int32_t *word, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_word, dim3(1), dim3(1), 0, stream, word);
    return hipGetLastError();
}

hipError_t launch_finalize(const FinArgs &a, hipStream_t stream)
{
    int npow = 1, kpow = 1;
    while (npow < a.S * a.kcap) npow <<= 1;
    while (kpow < (a.krs > a.k ? a.krs : a.k)) kpow <<= 1;
    if (npow > KNN_FIN_MAX || kpow > KNN_MAX_KCAP) return hipErrorInvalidValue;
    const size_t lds = (size_t)(npow + kpow) * sizeof(u64);
    hipLaunchKernelGGL(finalize_rows, dim3((unsigned)a.nq), dim3(64), lds, stream, a);
    return hipGetLastError();
}

}  // namespace knn
