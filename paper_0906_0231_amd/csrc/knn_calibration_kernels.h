// contract_only<SHAPE, DC>: calibration of two design choices of the fp32 tile kernels, which
// matrix instruction and how many coordinates per LDS step.  It is knn_tiles_qreg's contraction
// and nothing else -- 4 waves, a wave = 32 queries whose operands stay in registers (d = 256),
// 64 reference rows staged through double-buffered, swizzled LDS DC coordinates at a time, one
// barrier per step, no selection -- with
//   SHAPE 0: v_mfma_f32_32x32x2_f32, two 32x32 accumulator blocks per wave (the kernels' choice),
//   SHAPE 1: v_mfma_f32_16x16x4_f32, eight 16x16 blocks per wave,
//   DC = 16, 32 (the kernels' choice) or 64 coordinates per step.
// The reference rows are the same 64 x 256 block for every tile (an L2-resident stream, as the
// shared reference stream of the real kernels mostly is).  Included by knn_kernels.hip only.
#ifndef KNN_CALIBRATION_KERNELS_H_
#define KNN_CALIBRATION_KERNELS_H_

namespace knn {

// XOR swizzle of the 16-byte units of a staged row (DC/4 units per row): a row is stored
// contiguously, and 16 consecutive rows reading the same logical unit fall into different banks
template <int DC>
__device__ __forceinline__ int cal_swz(int row)
{
    if (DC == 16) return (row >> 2) & 3;           // 64-byte rows: four rows share a 256-byte line of banks
    if (DC == 32) return (row & 7) ^ ((row >> 3) & 1);
    return row & 15;                               // 256-byte rows: every row starts at bank 0
}

template <int SHAPE, int DC>
__global__ __launch_bounds__(256, 2) void contract_only(const float *R, int64_t tiles, float *sink)
{
    constexpr int D = 256;
    constexpr int NK = D / DC;                     // steps per tile
    constexpr int U = DC / 4;                      // 16-byte units per staged row
    constexpr int UPT = 64 * U / 256;              // units a thread stages per step
    __shared__ __attribute__((aligned(16))) float sr[2][64 * DC];
    const int tid = threadIdx.x;
    const int lane = tid & 63;

    // query operands: D/2 floats per lane, busy mantissas, both signs, small so that sums stay bounded
    f32x4 qreg[D / 8];
    uint32_t hsh = (blockIdx.x * 256u + tid) * 2654435761u + 99u;
#pragma unroll
    for (int i = 0; i < D / 8; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            hsh = hsh * 1664525u + 1013904223u;
            qreg[i][e] = __uint_as_float(0x3a000000u | (hsh >> 9)) * ((hsh & 256u) ? 1.f : -1.f);
        }

    f32x4 g[UPT];
    auto issue = [&](int kc) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            const int u = tid + 256 * i, row = u / U, unit = u % U;
            g[i] = *(const f32x4 *)(R + row * D + kc * DC + unit * 4);
        }
    };
    auto stash = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            const int u = tid + 256 * i, row = u / U, unit = u % U;
            *(f32x4 *)&sr[buf][row * DC + ((unit ^ cal_swz<DC>(row)) << 2)] = g[i];
        }
    };

    f32x16 acc32[2];
    f32x4 acc16[8];
#pragma unroll
    for (int i = 0; i < 2; ++i) acc32[i] = f32x16{};
#pragma unroll
    for (int i = 0; i < 8; ++i) acc16[i] = f32x4{};

    issue(0);
    stash(0);
    __syncthreads();
    int buf = 0;
    auto step = [&](auto kc_tag, int) __attribute__((always_inline)) {
        constexpr int kc = decltype(kc_tag)::value;
        issue((kc + 1) % NK);
        __builtin_amdgcn_sched_barrier(0);
        const float *rb = &sr[buf][0];
        if (SHAPE == 0) {
            // lane (ql, h): rows ql and 32 + ql, coordinates 8s + 4h .. + 3 of every slab of 8
            const int ql = lane & 31, h = lane >> 5, sw = cal_swz<DC>(ql);
#pragma unroll
            for (int s = 0; s < DC / 8; ++s) {
                const int off = ((2 * s + h) ^ sw) << 2;
                const f32x4 rf0 = *(const f32x4 *)(rb + ql * DC + off);
                const f32x4 rf1 = *(const f32x4 *)(rb + (32 + ql) * DC + off);
                const f32x4 qf = qreg[kc * (DC / 8) + s];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    acc32[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(rf0[c], qf[c], acc32[0], 0, 0, 0);
                    acc32[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(rf1[c], qf[c], acc32[1], 0, 0, 0);
                }
            }
        } else {
            // lane (r16, kq): rows r16 + 16 t, coordinates 16 g + 4 kq .. + 3 of every group of 16;
            // query block b of the wave uses registers 2 (16-coordinate group) + b
            const int r16 = lane & 15, kq = lane >> 4, sw = cal_swz<DC>(r16);
#pragma unroll
            for (int gi = 0; gi < DC / 16; ++gi) {
                const int off = ((4 * gi + kq) ^ sw) << 2;
                f32x4 rf[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) rf[t] = *(const f32x4 *)(rb + (r16 + 16 * t) * DC + off);
                const f32x4 q0 = qreg[(kc * (DC / 16) + gi) * 2], q1 = qreg[(kc * (DC / 16) + gi) * 2 + 1];
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        acc16[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(rf[t][c], q0[c], acc16[t], 0, 0, 0);
                        acc16[4 + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(rf[t][c], q1[c], acc16[4 + t], 0, 0, 0);
                    }
            }
        }
        stash(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    };
    for (int64_t t = 0; t < tiles; ++t) for_each_step<NK>(step, 0);

    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) sum += acc32[i][e];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) sum += acc16[i][e];
    sink[(int64_t)blockIdx.x * 256 + tid] = sum;
}

}  // namespace knn

#endif
