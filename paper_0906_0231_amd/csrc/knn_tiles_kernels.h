// The fused distance + selection kernels of the full-square schedule on the fp32 matrix cores
// (paper Sect. 5 and 6 in one pass): knn_tiles (streaming, any d) and knn_tiles_qreg (query
// operands in registers, d <= 256).  Included by knn_kernels.hip only.
#ifndef KNN_TILES_KERNELS_H_
#define KNN_TILES_KERNELS_H_

namespace knn {

// ---------------------------------------------------------------------------
// knn_tiles: the fused kernel.
//
// Workgroup = 4 waves, tile = 128 queries x 128 references, d consumed DC
// coordinates at a time through double-buffered LDS.  Wave w owns queries
// 32w..32w+31 of the tile against all 128 references: four 32x32 accumulator
// blocks of v_mfma_f32_32x32x2_f32 with the QUERY on the lane axis (B operand)
// and the reference on the register axis (A operand).  So lane l (and l+32) holds
// every distance of query l%32 in its own registers, the query's threshold lives
// in one VGPR, and the common case of the selection -- nothing in the tile beats
// the current k-th best -- is a min-reduction over the lane's own registers and one
// compare, with no cross-lane traffic.  Survivors go to a small per-query queue
// in LDS and are merged into the query's sorted k-list by the whole wave.
//
// A workgroup keeps its query tile for a whole slice of the reference range, so
// a query's list and threshold are private to one wave: no atomics on global
// memory, no locks.  The paper gives each GPU private heaps for the same reason
// (Sect. 4); here the unit is a wave.
// ---------------------------------------------------------------------------
constexpr int TQ = 128;
constexpr int TR = 128;
constexpr int DC = KNN_DC;
constexpr int LSTR = DC + 4;    // LDS row stride (floats): 16-byte aligned rows, conflict-free b128 reads
constexpr int QCAP = 16;        // queue slots per query
constexpr int NSLAB = DC / 8;
constexpr int LD_PER_ROW = DC / 4;            // float4 loads per staged row
constexpr int ROWS_PER_PASS = 256 / LD_PER_ROW;
constexpr int NPASS = TQ / ROWS_PER_PASS;

struct __attribute__((aligned(16))) TileSmem {
    float q[2][TQ * LSTR];
    float r[2][TR * LSTR];
    float c[2][TR];
    u64 cq[4][32][QCAP];
    uint32_t cnt[4][32];
};


__global__ __launch_bounds__(256, 2) void knn_tiles(TileArgs a)
{
    __shared__ TileSmem sm;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int h = lane >> 5;
    const int ql = lane & 31;

    const int qt = blockIdx.x / a.S;
    const int split = blockIdx.x - qt * a.S;
    const int64_t qbase = (int64_t)qt * TQ;
    const int rt0 = split * a.rt_per_split;
    const int rt1 = min(rt0 + a.rt_per_split, a.n_rtiles);
    const int nk = a.dpad / DC;

    // this wave's 32 lists
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

    // staging: thread -> (row, 16-byte column) of the DC-wide chunk
    const int lcol = (tid % LD_PER_ROW) * 4;
    const int lrow = tid / LD_PER_ROW;
    const float *qsrc[NPASS];
#pragma unroll
    for (int i = 0; i < NPASS; ++i) {
        int64_t row = min(qbase + lrow + i * ROWS_PER_PASS, a.nq - 1);
        qsrc[i] = a.Qp + row * a.ldq + lcol;
    }
    f32x4 gq[NPASS], gr[NPASS];
    float gc = 0.f;

    // the reference rows' addresses are worked out once per tile (64-bit multiplies: a step has
    // 2048 matrix-pipe cycles per wave, and vector instructions do not hide behind them)
    const float *rsrc[NPASS];
    auto issue = [&](int rt, int kc) __attribute__((always_inline)) {
        if (kc == 0) {
#pragma unroll
            for (int i = 0; i < NPASS; ++i) {
                int64_t row = min((int64_t)rt * TR + lrow + i * ROWS_PER_PASS, a.nr - 1);
                rsrc[i] = a.Rp + row * a.ldr + lcol;
            }
            if (tid < TR) gc = a.cR[(int64_t)rt * TR + tid];
        }
#pragma unroll
        for (int i = 0; i < NPASS; ++i) {
            gq[i] = *(const f32x4 *)(qsrc[i] + kc * DC);
            gr[i] = *(const f32x4 *)(rsrc[i] + kc * DC);
        }
    };
    auto stash = [&](int buf, int kc) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NPASS; ++i) {
            *(f32x4 *)&sm.q[buf][(lrow + i * ROWS_PER_PASS) * LSTR + lcol] = gq[i];
            *(f32x4 *)&sm.r[buf][(lrow + i * ROWS_PER_PASS) * LSTR + lcol] = gr[i];
        }
        if (kc == 0 && tid < TR) sm.c[buf][tid] = gc;
    };

    f32x16 acc[4];
    const int total = (rt1 - rt0) * nk;
    if (total > 0) {
        issue(rt0, 0);
        stash(0, 0);
    }
    __syncthreads();

    int rt = rt0, kc = 0;
    for (int it = 0; it < total; ++it) {
        const int buf = it & 1;
        int nrt = rt, nkc = kc + 1;
        if (nkc == nk) { nkc = 0; nrt = rt + 1; }
        // the last step fetches its own operands again instead of nothing: fetch and deposit are
        // unconditional, so the compiler knows at the top of a step that no load is pending
        if (it + 1 == total) { nrt = rt; nkc = kc; }
        issue(nrt, nkc);

        if (kc == 0) {
            // accumulators start at c_j: register r of block t is reference row 32t + 8(r/4) + 4h + r%4
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 cv = *(const f32x4 *)&sm.c[buf][t * 32 + g * 8 + h * 4];
                    acc[t][4 * g + 0] = cv[0];
                    acc[t][4 * g + 1] = cv[1];
                    acc[t][4 * g + 2] = cv[2];
                    acc[t][4 * g + 3] = cv[3];
                }
        }
        {
            const float *qp = &sm.q[buf][(32 * w + ql) * LSTR + h * 4];
            const float *rp = &sm.r[buf][ql * LSTR + h * 4];
#pragma unroll
            for (int s = 0; s < NSLAB; ++s) {
                // lane half h supplies coordinates 8s+4h .. 8s+4h+3; MFMA number c
                // contracts the coordinate pair (8s+c, 8s+4+c) -- the same pairing
                // for both operands, so the sum over d is complete and unchanged.
                f32x4 qf = *(const f32x4 *)(qp + s * 8);
                f32x4 rf[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) rf[t] = *(const f32x4 *)(rp + t * 32 * LSTR + s * 8);
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(rf[t][c], qf[c], acc[t], 0, 0, 0);
            }
        }

        if (kc == nk - 1) {
            // ---- selection on the accumulators (Sect. 6: test against the current
            // k-th smallest first, since for k << n almost everything is discarded) ----
            __builtin_amdgcn_s_setprio(1);
            float m4 = min16(acc[0]);
            m4 = fminf(m4, min16(acc[1]));
            m4 = fminf(m4, min16(acc[2]));
            m4 = fminf(m4, min16(acc[3]));
            if (__ballot(m4 <= st.tau_p)) {
                // a copy, so that the address of the hot loop's accumulators is never taken
                f32x16 blocks[4] = {acc[0], acc[1], acc[2], acc[3]};
                select_rare<4, QCAP>(blocks, rt * TR + 4 * h, a.nr, a.kcap, a.k, st, lane);
            }
            __builtin_amdgcn_s_setprio(0);
        }

        stash(buf ^ 1, nkc);
        __syncthreads();
        rt = nrt;
        kc = nkc;
    }
    merge_queues<QCAP>(st, a.kcap, a.k, lane);
}

// ---------------------------------------------------------------------------
// knn_tiles_qreg<DPAD>: the fused kernel with the query tile stationary in REGISTERS.
//
// Same ownership as knn_tiles (4 waves, wave = 32 queries, two independent workgroups
// per CU), but a wave loads the B operands of its 32 queries for all DPAD coordinates
// once per sweep: lane (q, h) keeps coordinates 8s+4h .. 8s+4h+3 of every 8-wide slab s,
// DPAD/2 floats per lane (128 VGPRs at d = 256).  Only reference rows are staged through
// LDS (64 rows x 32 coordinates per step, two 32x32 accumulator blocks per wave), so per
// reference row the workgroup reads d floats instead of 2d, the 64 workgroups of an XCD
// all stream the same reference rows through the L2, and no query tile competes for it.
// The d-loop is fully unrolled so that the query registers are addressed statically.
// ---------------------------------------------------------------------------
// Calls f(integral_constant<int, 0>, x), ..., f(integral_constant<int, N-1>, x): a loop whose
// counter is a compile-time constant inside the body.
template <typename F, int... I>
__device__ __forceinline__ void for_each_step_impl(F &f, int x, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}, x), ...);
}
template <int N, typename F>
__device__ __forceinline__ void for_each_step(F &f, int x)
{
    for_each_step_impl(f, x, std::make_integer_sequence<int, N>{});
}

constexpr int QG_TR = 64;                         // reference rows per tile
constexpr int QG_DC = 32;                         // coordinates per step
constexpr int QG_NSLAB = QG_DC / 8;
constexpr int QG_RBUF = QG_TR * QG_DC;            // floats per staging buffer (128-byte rows)

// 128-byte rows of eight 16-byte units, XOR-swizzled: a row is stored contiguously, and
// 16 consecutive rows reading the same logical unit touch 16 different bank groups.
__device__ __forceinline__ int qg_swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

struct __attribute__((aligned(16))) QregSmem {
    float r[2][QG_RBUF];
    float c[2][QG_TR];
    u64 cq[4][32][QCAP];
    uint32_t cnt[4][32];
};

// SHARE: the reference range is cut into slices that run side by side, each with its own list
// per query starting empty.  A slice's k-th best is an upper bound of the final k-th best, so the
// slices publish theirs (atomic minimum on one word per query) and test against the smallest
// published so far; a stale read is merely looser.  Matters when n is small against k (the
// shape of the paper's Table 1: without it 40 % of all pairs entered a queue at n = 10 000).
// SUBSET: the queries are a compacted subset whose size is only known on the device (a.nq_dev;
// a.nq is its capacity) and whose self indices come from a table (a.self_rows): the second pass
// of the split-precision plan over the rows its filter could not certify.  Workgroups beyond the
// subset leave at once.
template <int DPAD, bool SHARE, bool SUBSET = false>
__global__ __launch_bounds__(256, 2) void knn_tiles_qreg(TileArgs a)
{
    constexpr int NK = DPAD / QG_DC;
    constexpr int NS = DPAD / 8;
    __shared__ QregSmem sm;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int h = lane >> 5;
    const int ql = lane & 31;

    const int qt = blockIdx.x / a.S;
    const int split = blockIdx.x - qt * a.S;
    const int64_t qbase = (int64_t)qt * TQ;
    if (SUBSET) {
        a.nq = min(a.nq, (int64_t)*a.nq_dev);
        if (qbase >= a.nq) return;                // the whole workgroup, before any barrier
    }
    // slices are cut in units of 128 reference rows; this kernel walks them 64 at a time
    const int rt0 = split * a.rt_per_split * 2;
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
    if (SUBSET) st.selfj = qvalid ? a.self_rows[myq] : -1;
    st.Lw = Lw;
    st.cq = &sm.cq[w][0][0];
    st.cnt = &sm.cnt[w][0];
    st.mine = 0;
    uint32_t *mybound = SHARE ? a.bound + min(myq, a.nq - 1) : nullptr;
    uint32_t seen = 0xffffffffu;

    // the wave's query operands, once
    f32x4 qreg[NS];
    {
        const float *qrow = a.Qp + min(myq, a.nq - 1) * a.ldq + h * 4;
#pragma unroll
        for (int s = 0; s < NS; ++s) qreg[s] = *(const f32x4 *)(qrow + s * 8);
    }

    // staging of the 64 reference rows: thread -> 16-byte unit lunit of rows lrow and lrow+32,
    // through registers (a direct global -> LDS deposit, global_load_lds_dwordx4, was measured
    // 3 % slower here)
    const int lrow = tid >> 3, lunit = tid & 7;
    const int st_off = lrow * QG_DC + ((lunit ^ qg_swz(lrow)) << 2);   // rows r and r+32 swizzle alike
    f32x4 g0, g1;
    float gc = 0.f;
    auto issue = [&](int rt, int kc) __attribute__((always_inline)) {
        int64_t r0 = min((int64_t)rt * QG_TR + lrow, a.nr - 1);
        int64_t r1 = min((int64_t)rt * QG_TR + lrow + 32, a.nr - 1);
        g0 = *(const f32x4 *)(a.Rp + r0 * a.ldr + kc * QG_DC + lunit * 4);
        g1 = *(const f32x4 *)(a.Rp + r1 * a.ldr + kc * QG_DC + lunit * 4);
        if (kc == 0 && tid < QG_TR) gc = a.cR[(int64_t)rt * QG_TR + tid];
    };
    auto stash = [&](int buf, int kc) __attribute__((always_inline)) {
        *(f32x4 *)&sm.r[buf][st_off] = g0;
        *(f32x4 *)&sm.r[buf][st_off + 32 * QG_DC] = g1;
        if (kc == 0 && tid < QG_TR) sm.c[buf][tid] = gc;
    };
    // fragment read offsets: block t (rows 32t + ql), slab s -> unit 2s + h
    const int rbase0 = ql * QG_DC, rbase1 = (32 + ql) * QG_DC;
    const int sw = qg_swz(ql);                    // rows ql and 32+ql swizzle alike

    f32x16 acc0, acc1;
    if (rt0 < rt1) {
        issue(rt0, 0);
        stash(0, 0);
    }
    __syncthreads();

    int buf = 0;
    // one step = QG_DC coordinates; kc is a compile-time constant so that qreg[] is
    // addressed statically (a run-time index would push the array to scratch memory)
    auto step = [&](auto kc_tag, int rt) __attribute__((always_inline)) {
        constexpr int kc = decltype(kc_tag)::value;
        constexpr bool last = kc == NK - 1;
        const bool more = !last || rt + 1 < rt1;
        if (more) issue(last ? rt + 1 : rt, last ? 0 : kc + 1);
        // keep the loads up here: their latency must overlap this step's matrix work
        __builtin_amdgcn_sched_barrier(0);
        if (kc == 0) {
            // what the other slices have reached: requested now, used after the tile
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
        for (int s = 0; s < QG_NSLAB; ++s) {
            const int u = ((2 * s + h) ^ sw) << 2;
            f32x4 rf0 = *(const f32x4 *)(rb + rbase0 + u);
            f32x4 rf1 = *(const f32x4 *)(rb + rbase1 + u);
            const f32x4 qf = qreg[kc * QG_NSLAB + s];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(rf0[c], qf[c], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(rf1[c], qf[c], acc1, 0, 0, 0);
            }
        }
        if (last) {
            // short vector work at raised priority: it does not queue behind the other
            // workgroup's matrix instructions on this SIMD (measured: -0.3 to -1.5 %)
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

}  // namespace knn

#endif
