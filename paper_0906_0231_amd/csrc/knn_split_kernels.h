// Split-precision experiment: the fused full-square kernel with both operands cut into two bf16
// pieces and the contraction done by three bf16 matrix products per pair (hi*hi, hi*lo, lo*hi)
// on v_mfma_f32_32x32x16_bf16 -- 16 times the rate of the fp32 matrix instruction for 3 times the
// products.  What it computes is an APPROXIMATION p~ of the selection value p = |r|^2 - 2 q.r
// with a known error bound, so it is used as a filter: every query keeps the K' > k references
// of smallest p~, finalize_rows prices those K' exactly (double, from the original rows), takes
// the k best, and proves from the bound that nothing left out can belong (see finalize_rows).
// Included by knn_kernels.hip only.
#ifndef KNN_SPLIT_KERNELS_H_
#define KNN_SPLIT_KERNELS_H_

namespace knn {

// fp32 -> bf16, round to nearest even (inputs are finite)
__device__ __forceinline__ uint32_t bf16_rne(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_value(uint32_t b) { return __uint_as_float(b << 16); }

// ---------------------------------------------------------------------------
// prep_split: one wave per row.  Writes the row scaled by `scale` (a power of two: -2 for the
// query side, 1 for the reference side, so that the scaling is exact) as two bf16 pieces,
//   hi = bf16(v),  lo = bf16(v - hi)      (v - hi is exact in fp32; |v - hi - lo| <= 2^-16 |v|)
// in the order the kernel's 16-byte operand reads want: a row is dpad 4-byte words; the 32
// words of coordinate chunk kc hold the 32 hi pieces of coordinates 32 kc .. 32 kc + 31 (two per
// word, ascending) and then their 32 lo pieces.  A row thus takes 4 dpad bytes, as in fp32, and
// is staged through LDS by the same code.  Also c_j = |x_j|^2 (+inf beyond n), accumulated in
// double and rounded once, and the plain squared norm for finalize.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prep_split(SplitPrepArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    if (a.c_out) {
        int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
        if (g < a.n_cpad - a.n) a.c_out[a.n + g] = __builtin_inff();
    }
    for (int64_t row = wave; row < a.n; row += nwaves) {
        const float *x = a.X + row * (int64_t)a.d;
        uint32_t *o = a.out + row * (int64_t)a.dpad;
        for (int wd = lane; wd < a.dpad; wd += 64) {
            const int chunk = wd >> 5, w = wd & 31;
            const int c0 = chunk * 32 + 2 * (w & 15);
            auto val = [&](int c) __attribute__((always_inline)) {
                return a.mu != nullptr ? (float)((double)x[c] - (double)a.mu[c]) : x[c];
            };
            const float v0 = c0 < a.d ? a.scale * val(c0) : 0.f;
            const float v1 = c0 + 1 < a.d ? a.scale * val(c0 + 1) : 0.f;
            uint32_t b0 = bf16_rne(v0), b1 = bf16_rne(v1);
            if (w >= 16) {
                b0 = bf16_rne(v0 - bf16_value(b0));
                b1 = bf16_rne(v1 - bf16_value(b1));
            }
            o[wd] = b0 | (b1 << 16);
        }
        if (a.c_out || a.s_out) {
            // of the value the pieces are cut from (the centred one, rounded to fp32)
            double s = 0.0;
            for (int c = lane; c < a.d; c += 64) {
                const double v = a.mu != nullptr ? (double)(float)((double)x[c] - (double)a.mu[c]) : (double)x[c];
                s = fma(v, v, s);
            }
            s = wave_sum_f64(s);
            if (lane == 0) {
                if (a.c_out) a.c_out[row] = (float)s;
                if (a.s_out) a.s_out[row] = (float)s;
            }
        }
        if (a.b_out && lane == 0) a.b_out[row] = 0xffffffffu;
    }
}

// ---------------------------------------------------------------------------
// knn_tiles_split<DPAD, WAVES, SHARE>: knn_tiles_qreg's structure -- a wave owns 32 queries whose
// operands stay in registers for the whole sweep, reference rows are staged through LDS 64 rows x
// 32 coordinates at a time, the selection runs on the accumulators -- with bf16 pieces:
//   per 16 coordinates and 32x32 block:  acc += rh*qh;  acc += rh*ql;  acc += rl*qh
// (the lo*lo product, <= 2^-16 of the term, is left to the error bound).  Lane (q, h) keeps, per
// chunk of 32 coordinates, the hi and lo pieces of coordinates 16 s + 8 h .. + 7 for s = 0, 1:
// DPAD/2 registers in all, as in fp32.  One step has 12 matrix instructions of 32 cycles per wave
// where the fp32 kernel has 32 of 64 cycles, for the same 8 KB of reference rows, so the
// workgroup is WAVES = 8 waves (256 queries) to halve the reference traffic per pair.
// The lists keep a.k = K' entries each (all live); see finalize_rows for what happens to them.
// Measured at n = 2^20, d = 256: 1.30 s, of which the selection's rare path 10 %; with the matrix
// instructions taken out the rest still takes 0.82 s, with the loads taken out 0.99 s.  None of
// these changed that by more than +-2 %: two chunks per barrier, two query blocks per wave (half
// the LDS reads), reference rows requested two steps ahead (straight into LDS, or through a second
// register set), fragment reads one sub-step ahead of their matrix instructions with the barrier
// in mid-step.  Matrix instructions alone
// (mfma_bf16_only) sustain 1.89e15 flop/s on this device, 0.76 of the nominal peak.
// ---------------------------------------------------------------------------
template <int WAVES>
struct __attribute__((aligned(16))) SplitSmem {
    float r[2][QG_RBUF];
    float c[2][QG_TR];
    u64 cq[WAVES][32][QCAP];
    uint32_t cnt[WAVES][32];
};

template <int DPAD, int WAVES, bool SHARE>
__global__ __launch_bounds__(64 * WAVES, 2) void knn_tiles_split(TileArgs a)
{
    constexpr int NK = DPAD / QG_DC;
    constexpr int NT = 64 * WAVES;                // threads
    constexpr int UPT = 512 / NT;                 // 16-byte units a thread stages per step (2 or 1)
    constexpr int RPP = 64 / UPT;                 // rows per staging pass
    __shared__ SplitSmem<WAVES> sm;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int h = lane >> 5;
    const int ql = lane & 31;

    const int qt = blockIdx.x / a.S;
    const int split = blockIdx.x - qt * a.S;
    const int64_t qbase = (int64_t)qt * (32 * WAVES);
    const int rt0 = split * a.rt_per_split * 2;   // slices are cut in units of 128 reference rows
    const int rt1 = min(rt0 + a.rt_per_split * 2, (int)((a.nr + QG_TR - 1) / QG_TR));

    u64 *Lw = a.lists + ((int64_t)split * a.nq_pad + qbase + 32 * w) * a.kcap;
    for (int i = lane; i < 32 * a.kcap; i += 64) Lw[i] = KEY_INF;
    if (lane < 32) sm.cnt[w][lane] = 0;

    const int64_t myq = qbase + 32 * w + ql;
    const bool qvalid = myq < a.nq;
    SelState st;
    st.tau_key = qvalid ? KEY_INF : 0ull;
    st.tau_p = qvalid ? __builtin_inff() : -__builtin_inff();
    st.selfj = (a.self_offset >= 0 && qvalid) ? (int32_t)(a.self_offset + myq) : -1;
    st.Lw = Lw;
    st.cq = &sm.cq[w][0][0];
    st.cnt = &sm.cnt[w][0];
    st.mine = 0;
    uint32_t *mybound = SHARE ? a.bound + min(myq, a.nq - 1) : nullptr;
    uint32_t seen = 0xffffffffu;

    // the wave's query operands, once: [chunk][s] hi and lo pieces
    bf16x8 qh[NK * 2], ql8[NK * 2];
    {
        const float *qrow = a.Qp + min(myq, a.nq - 1) * a.ldq + h * 4;
#pragma unroll
        for (int kc = 0; kc < NK; ++kc)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                qh[kc * 2 + s] = __builtin_bit_cast(bf16x8, *(const f32x4 *)(qrow + kc * 32 + s * 8));
                ql8[kc * 2 + s] = __builtin_bit_cast(bf16x8, *(const f32x4 *)(qrow + kc * 32 + 16 + s * 8));
            }
    }

    // staging of the 64 reference rows (128 bytes each per step): thread -> 16-byte unit lunit
    // of row lrow (and of row lrow + 32 when there are 256 threads)
    const int lrow = tid >> 3, lunit = tid & 7;
    const int st_off = lrow * QG_DC + ((lunit ^ qg_swz(lrow)) << 2);   // rows r and r+32 swizzle alike
    f32x4 g[UPT];
    float gc = 0.f;
    auto issue = [&](int rt, int kc) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            int64_t r = min((int64_t)rt * QG_TR + lrow + i * RPP, a.nr - 1);
            g[i] = *(const f32x4 *)(a.Rp + r * a.ldr + kc * QG_DC + lunit * 4);
        }
        if (kc == 0 && tid < QG_TR) gc = a.cR[(int64_t)rt * QG_TR + tid];
    };
    auto stash = [&](int buf, int kc) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) *(f32x4 *)&sm.r[buf][st_off + i * RPP * QG_DC] = g[i];
        if (kc == 0 && tid < QG_TR) sm.c[buf][tid] = gc;
    };
    const int rbase0 = ql * QG_DC, rbase1 = (32 + ql) * QG_DC;
    const int sw = qg_swz(ql);                    // rows ql and 32+ql swizzle alike

    f32x16 acc0, acc1;
    if (rt0 < rt1) {
        issue(rt0, 0);
        stash(0, 0);
    }
    __syncthreads();

    int buf = 0;
    auto step = [&](auto kc_tag, int rt) __attribute__((always_inline)) {
        constexpr int kc = decltype(kc_tag)::value;
        constexpr bool last = kc == NK - 1;
        const bool more = !last || rt + 1 < rt1;
        if (more) issue(last ? rt + 1 : rt, last ? 0 : kc + 1);
        __builtin_amdgcn_sched_barrier(0);
        if (kc == 0) {
            if (SHARE) seen = __hip_atomic_load(mybound, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                f32x4 c0 = *(const f32x4 *)&sm.c[buf][gg * 8 + h * 4];
                f32x4 c1 = *(const f32x4 *)&sm.c[buf][32 + gg * 8 + h * 4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc0[4 * gg + e] = c0[e];
                    acc1[4 * gg + e] = c1[e];
                }
            }
        }
        const float *rb = &sm.r[buf][0];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int uh = ((2 * s + h) ^ sw) << 2, ul = ((4 + 2 * s + h) ^ sw) << 2;
            const bf16x8 rh0 = __builtin_bit_cast(bf16x8, *(const f32x4 *)(rb + rbase0 + uh));
            const bf16x8 rh1 = __builtin_bit_cast(bf16x8, *(const f32x4 *)(rb + rbase1 + uh));
            const bf16x8 rl0 = __builtin_bit_cast(bf16x8, *(const f32x4 *)(rb + rbase0 + ul));
            const bf16x8 rl1 = __builtin_bit_cast(bf16x8, *(const f32x4 *)(rb + rbase1 + ul));
            const bf16x8 xh = qh[kc * 2 + s], xl = ql8[kc * 2 + s];
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rh0, xh, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rh1, xh, acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rh0, xl, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rh1, xl, acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rl0, xh, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rl1, xh, acc1, 0, 0, 0);
        }
        if (last) {
            __builtin_amdgcn_s_setprio(1);
            float m2 = fminf(min16(acc0), min16(acc1));
            if (SHARE && seen != 0xffffffffu) st.tau_p = fminf(st.tau_p, ord2f(seen));
            if (__ballot(m2 <= st.tau_p)) {
                f32x16 blocks[2] = {acc0, acc1};
                select_rare<2, QCAP>(blocks, rt * QG_TR + 4 * h, a.nr, a.kcap, a.k, st, lane);
                if (SHARE && h == 0 && qvalid && st.tau_key != KEY_INF)
                    atomicMin(mybound, (uint32_t)(st.tau_key >> 32));
            }
            __builtin_amdgcn_s_setprio(0);
        }
        if (more) stash(buf ^ 1, last ? 0 : kc + 1);
        __syncthreads();
        buf ^= 1;
    };
    for (int rt = rt0; rt < rt1; ++rt) for_each_step<NK>(step, rt);
    merge_queues<QCAP>(st, a.kcap, a.k, lane);
}

// ---------------------------------------------------------------------------
// mfma_bf16_only: calibration.  Nothing but v_mfma_f32_32x32x16_bf16 on NACC independent
// accumulators per wave (4; 2 is the dependency pattern of knn_tiles_split with one query
// block per wave), busy operands, no memory traffic in the loop: the bf16 matrix rate the
// device sustains under load, clock included.
// ---------------------------------------------------------------------------
template <int NACC>
__global__ __launch_bounds__(256) void mfma_bf16_only(int64_t groups_of_16, float *sink)
{
    f32x16 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = f32x16{};
    bf16x8 x[4], y[4];
    uint32_t hsh = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        f32x4 xv, yv;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // two bf16 values per word: magnitudes in [0.5, 1), both signs; y scaled down so that sums stay bounded
            hsh = hsh * 1664525u + 1013904223u;
            xv[e] = __uint_as_float((0x3f003f00u | (hsh & 0x007f007fu)) ^ (hsh & 0x80008000u));
            hsh = hsh * 1664525u + 1013904223u;
            yv[e] = __uint_as_float((0x35003500u | (hsh & 0x007f007fu)) ^ (hsh & 0x80008000u));
        }
        x[u] = __builtin_bit_cast(bf16x8, xv);
        y[u] = __builtin_bit_cast(bf16x8, yv);
    }
    for (int64_t i = 0; i < groups_of_16; ++i) {
#pragma unroll
        for (int u = 0; u < 16 / NACC; ++u)
#pragma unroll
            for (int c = 0; c < NACC; ++c)
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[(u + c) & 3], y[(u + (c >> 1)) & 3], acc[c], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int c = 0; c < NACC; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) t += acc[c][e];
    sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = t;
}

}  // namespace knn

#endif
