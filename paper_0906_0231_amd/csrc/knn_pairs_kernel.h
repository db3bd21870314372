// The symmetric schedule (paper Sect. 3-4: each unordered pair once, both rows updated).
// Included by knn_kernels.hip only.
#ifndef KNN_PAIRS_KERNEL_H_
#define KNN_PAIRS_KERNEL_H_

namespace knn {

// ---------------------------------------------------------------------------
// knn_pairs_qreg<DPAD>: the symmetric schedule (Sect. 3-4 of the paper: delta(u,v) =
// delta(v,u), so each unordered pair is evaluated once and pushed to both rows).
//
// Rows are cut into blocks of B.  One workgroup evaluates one unordered pair of blocks
// (a, b): every tile is used in both directions -- "direct": rows of a are the queries
// (lane axis), rows of b the references; "mirror": the same accumulator, read along the
// register axis, is a candidate for the list of reference row j with the query as its
// neighbour.  A launch is one round of a round-robin tournament over the blocks: its
// pairs are disjoint, so within a launch every row's list is touched by exactly one
// workgroup and ownership changes hands only at kernel boundaries.  No locks, no
// atomics on global memory; as in the paper the only synchronisation between
// workgroups is the return to the host queue (Sect. 2), and the work per launch is
// balanced by construction where the paper uses its zig-zag assignment (Sect. 4).
// round < 0 is the launch for the diagonal blocks (a, a): direct only, whole block.
//
// Mirror values: the accumulator is p = c_j + sum(Q'[q] R[j]); the row-j value of the
// same pair is p' = (p - c_j) + c_q.  The common-case test must not cost a pass over
// the registers per row, so it is one-sided: with T_j >= tau'_j + c_j + slack (the
// row's current k-th best plus its norm, rounded up generously) the lane keeps
// max_r (T_r - p_r) and compares it once with its own c_q; anything that could pass
// the exact test passes this one.  Survivors are tested exactly, queued per row in LDS
// and merged after the step barrier by the wave that serves the row.
// ---------------------------------------------------------------------------
constexpr int MQCAP = 8;                          // mirror queue slots per reference row of the tile

struct __attribute__((aligned(16))) PairSmem {
    float r[2][QG_RBUF];
    float c[2][QG_TR];
    float T[2][QG_TR];                            // one-sided mirror thresholds
    u64 mtau[2][QG_TR];                           // exact k-th best keys of the tile's reference rows
    u64 cq[4][32][QCAP];
    u64 mq[2][QG_TR][MQCAP];                      // mirror queues, by tile parity
    uint32_t cnt[4][32];
    uint32_t mcnt[2][QG_TR];
    uint32_t movf[2];                             // a mirror queue of the tile overflowed
    // per-thread selection state, parked here between epilogues so that it does not occupy
    // registers during the matrix loop (the d = 256 instance is at the 256-register limit)
    u64 tkey[256];                                // threshold key of the thread's query
    float tp[256];                                // its distance part
    float cqv[256];                               // c of the thread's query (+inf: no valid query)
    uint32_t taken[256];                          // mirror entries of the current tile: still without a slot (mask scan) / already queued (walk)
};

__device__ __forceinline__ float mirror_T(u64 tkey, float cj, float cmax, float abound)
{
    if (tkey == KEY_INF) return __builtin_inff();
    if (tkey == 0ull) return -__builtin_inff();   // row past the end: nothing may pass
    float t = ord2f((uint32_t)(tkey >> 32));
    float slack = (fabsf(t) + cmax + abound) * 3.814697265625e-06f;   // 2^-18
    return (t + cj) + slack + slack;
}

// MASKSCAN: how the mirror candidates of a tile are collected once the cheap test has fired --
// per-lane bit masks and lowest-bit passes (true), or a walk over the 32 registers with one
// ballot each (false).  The mask version is several times cheaper per call, which matters
// while thresholds are loose (small n, early rounds), but at d = 256 its few extra live
// registers push spills into the matrix loop (+4.7 % at n = 2^20, -5 % at n = 2^18): the host
// picks the walk for d = 256 and large n.
// SPLIT: the split-precision experiment's form of the same schedule.  Operand rows are two bf16
// pieces per value in the layout of prep_split -- per chunk of 32 coordinates the 16-byte units
// h, 2+h hold the hi pieces and 4+h, 6+h the lo pieces that lane half h needs, i.e. the very
// units (2s+h, s = 0..3) the fp32 loop reads -- so staging, query registers, accumulator layout
// and everything the selection does are shared and only the matrix instructions differ: three
// v_mfma_f32_32x32x16_bf16 per 16 coordinates and block.  The lists then hold a.k = K' entries
// by approximate value, mirrored values included (see finalize_rows).
template <int DPAD, bool MASKSCAN, bool SPLIT = false>
__global__ __launch_bounds__(256, 2) void knn_pairs_qreg(PairArgs a)
{
    constexpr int NK = DPAD / QG_DC;
    constexpr int NS = DPAD / 8;
    __shared__ PairSmem sm;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int h = lane >> 5;
    const int ql = lane & 31;

    // ---- which pair of blocks ----
    int ba, bb;
    const bool diag = a.round < 0;
    if (diag) {
        ba = bb = blockIdx.x;
    } else {
        const int M = a.NBp, p = blockIdx.x;       // circle method: M even, rounds 0..M-2
        if (p == 0) {
            ba = M - 1;
            bb = a.round;
        } else {
            ba = (a.round + p) % (M - 1);
            bb = (a.round - p + (M - 1)) % (M - 1);
        }
    }
    if (ba >= a.NB || bb >= a.NB) return;          // the dummy block of an odd count (whole workgroup)
    const int64_t qrow0 = (int64_t)ba * a.B, rrow0 = (int64_t)bb * a.B;
    const int nq_rows = (int)min((int64_t)a.B, a.n - qrow0);
    const int nr_rows = (int)min((int64_t)a.B, a.n - rrow0);
    const int n_qt = (nq_rows + TQ - 1) / TQ;
    const int n_rt = (nr_rows + QG_TR - 1) / QG_TR;
    const float cmax = *a.cmax;
    const float abound = a.metric == 1 ? 1.5f : 3.f * cmax;

    if (lane < 32) sm.cnt[w][lane] = 0;
    if (tid < 2 * QG_TR) sm.mcnt[tid >> 6][tid & 63] = 0;
    if (tid < 2) sm.movf[tid] = 0;

    // Staging of the 64 reference rows, global -> LDS without passing through registers
    // (global_load_lds_dwordx4: lane l of a wave deposits its 16 bytes at LDS base + 16 l;
    // this instance has no registers to spare for staging).  Wave w fills rows 8w..8w+7 and
    // 32+8w..32+8w+7; slot l of a 1 KB block is row l/8, physical unit l%8, so the lane
    // fetches the logical unit that the swizzle puts there.
    const int lrow = tid >> 3;
    const int lunit = (tid & 7) ^ qg_swz(lrow);   // rows r and r+32 swizzle alike
    const int rbase0 = ql * QG_DC, rbase1 = (32 + ql) * QG_DC;
    const int sw = qg_swz(ql);

    float gc = 0.f;
    u64 gmt = 0;
    auto issue = [&](int rt, int kc, int buf) __attribute__((always_inline)) {
        int64_t r0 = min(rrow0 + (int64_t)rt * QG_TR + lrow, a.n - 1);
        int64_t r1 = min(rrow0 + (int64_t)rt * QG_TR + lrow + 32, a.n - 1);
        lds_ptr d0 = (lds_ptr)&sm.r[buf][(w * 8) * QG_DC];
        lds_ptr d1 = (lds_ptr)&sm.r[buf][(32 + w * 8) * QG_DC];
        __builtin_amdgcn_global_load_lds(a.Rp + r0 * a.ldr + kc * QG_DC + lunit * 4, d0, 16, 0, 0);
        __builtin_amdgcn_global_load_lds(a.Rp + r1 * a.ldr + kc * QG_DC + lunit * 4, d1, 16, 0, 0);
        if (kc == 0 && tid < QG_TR) {
            int64_t row = rrow0 + (int64_t)rt * QG_TR + tid;     // < n_cpad: c is padded with +inf
            gc = a.cR[row];
            gmt = (!diag && row < a.n) ? a.lists[row * a.kcap + (a.k - 1)] : 0ull;
        }
    };
    // The per-tile arrays (c, T, mtau) alternate per tile (tb = tile parity), not per step: a
    // tile's mirror values are still needed after the next tile's first chunk has been staged.
    auto stash = [&](int kc, int tb) __attribute__((always_inline)) {
        if (kc == 0 && tid < QG_TR) {
            sm.c[tb][tid] = gc;
            sm.mtau[tb][tid] = gmt;
            sm.T[tb][tid] = mirror_T(gmt, gc, cmax, abound);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0): this step's deposits have landed
    };

    for (int qt = 0; qt < n_qt; ++qt) {
        const int64_t qbase = qrow0 + (int64_t)qt * TQ;
        const int64_t myq = qbase + 32 * w + ql;
        const bool qvalid = myq < a.n;
        {
            u64 *Lw = a.lists + (qbase + 32 * w) * a.kcap;
            if (diag)
                for (int i = lane; i < 32 * a.kcap; i += 64) Lw[i] = KEY_INF;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
            u64 tk = qvalid ? Lw[(int64_t)ql * a.kcap + (a.k - 1)] : 0ull;
            sm.tkey[tid] = tk;
            sm.tp[tid] = !qvalid ? -__builtin_inff() : tk == KEY_INF ? __builtin_inff() : ord2f((uint32_t)(tk >> 32));
            sm.cqv[tid] = qvalid ? a.cR[myq] : __builtin_inff();   // the query's own c, for the mirror values
        }
        auto load_state = [&]() __attribute__((always_inline)) {
            SelState st;
            st.tau_key = sm.tkey[tid];
            st.tau_p = sm.tp[tid];
            st.selfj = (diag && qvalid) ? (int32_t)myq : -1;
            st.Lw = a.lists + (qbase + 32 * w) * a.kcap;
            st.cq = &sm.cq[w][0][0];
            st.cnt = &sm.cnt[w][0];
            st.mine = 0;
            return st;
        };
        auto save_state = [&](const SelState &st) __attribute__((always_inline)) {
            sm.tkey[tid] = st.tau_key;
            sm.tp[tid] = st.tau_p;
        };

        f32x4 qreg[NS];
        {
            const float *qrow = a.Qp + min(myq, a.n - 1) * a.ldq + h * 4;
#pragma unroll
            for (int s = 0; s < NS; ++s) qreg[s] = *(const f32x4 *)(qrow + s * 8);
        }

        f32x16 acc0, acc1;
        issue(0, 0, 0);
        stash(0, 0);
        __syncthreads();

        // Mirror candidates of one tile: cheap one-sided test per register, exact test for
        // survivors, per-row queue (by tile parity).  Entries that found no slot are recorded
        // in a per-lane bit mask, which is all a re-scan after an overflow looks at (the
        // accumulators themselves are only ever read here).
        auto mirror_scan = [&](int rt, bool fresh) __attribute__((always_inline)) {
            const int par = rt & 1;
            const float cq = sm.cqv[tid];
            float dmax = -__builtin_inff();
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                f32x4 t0 = *(const f32x4 *)&sm.T[par][gg * 8 + h * 4];
                f32x4 t1 = *(const f32x4 *)&sm.T[par][32 + gg * 8 + h * 4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    dmax = fmaxf(dmax, t0[e] - acc0[4 * gg + e]);
                    dmax = fmaxf(dmax, t1[e] - acc1[4 * gg + e]);
                }
            }
            if (__ballot(qvalid && dmax >= cq) == 0) {
                if (fresh) sm.taken[tid] = 0;
                return;
            }
            if constexpr (MASKSCAN) {
                // Which of the lane's 32 values may pass: a bit mask built with constant register
                // indices (a re-scan after an overflow takes up the bits that found no slot).  Then
                // passes in which every lane handles ITS lowest marked entry, different entries in
                // different lanes at once: as many passes as the busiest lane has candidates.
                uint32_t mask;
                if (fresh) {
                    mask = 0;
    #pragma unroll
                    for (int gg = 0; gg < 4; ++gg) {
                        f32x4 t0 = *(const f32x4 *)&sm.T[par][gg * 8 + h * 4];
                        f32x4 t1 = *(const f32x4 *)&sm.T[par][32 + gg * 8 + h * 4];
    #pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            mask |= t0[e] - acc0[4 * gg + e] >= cq ? 1u << (4 * gg + e) : 0u;
                            mask |= t1[e] - acc1[4 * gg + e] >= cq ? 1u << (16 + 4 * gg + e) : 0u;
                        }
                    }
                    if (!qvalid) mask = 0;
                } else {
                    mask = sm.taken[tid];
                }
                uint32_t deferred = 0;
    #pragma unroll 1
                for (int t = 0; t < 2; ++t) {
                    const f32x16 v = t == 0 ? acc0 : acc1;
                    uint32_t m16 = (mask >> (16 * t)) & 0xffffu;
    #pragma unroll 1
                    for (int pass = 0; pass < 16 && __ballot(m16 != 0); ++pass) {
                        const int r = m16 ? __builtin_ctz(m16) : 0;
                        float p = v[0];
    #pragma unroll
                        for (int e = 1; e < 16; ++e) p = r == e ? v[e] : p;
                        const int m = t * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                        if (m16 != 0 && sm.T[par][m] - p >= cq) {      // the threshold may have been refreshed
                            float p2 = (p - sm.c[par][m]) + cq;        // this pair seen from row m
                            u64 key = make_key(p2, (int32_t)myq);
                            if (key < sm.mtau[par][m]) {
                                uint32_t slot = atomicAdd(&sm.mcnt[par][m], 1u);
                                if (slot < (uint32_t)MQCAP)
                                    sm.mq[par][m][slot] = key;
                                else
                                    deferred |= 1u << (16 * t + r);    // no slot: again after the merge
                            }
                        }
                        m16 &= m16 - 1;
                    }
                }
                sm.taken[tid] = deferred;
                if (deferred) atomicOr(&sm.movf[par], 1u);
            } else {
                // walk: sm.taken holds the entries already queued, which a re-scan skips
                uint32_t taken = fresh ? 0u : sm.taken[tid];
                bool ovf = false;
#pragma unroll 1
                for (int t = 0; t < 2; ++t) {
                    const f32x16 v = t == 0 ? acc0 : acc1;
#pragma unroll 1
                    for (int r = 0; r < 16; ++r) {
                        const int m = t * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                        const uint32_t bit = 1u << (t * 16 + r);
                        const float p = v[r];
                        bool c = qvalid && !(taken & bit) && sm.T[par][m] - p >= cq;
                        if (__ballot(c)) {
                            if (c) {
                                float p2 = (p - sm.c[par][m]) + cq;      // this pair seen from row m
                                u64 key = make_key(p2, (int32_t)myq);
                                if (key < sm.mtau[par][m]) {
                                    uint32_t slot = atomicAdd(&sm.mcnt[par][m], 1u);
                                    if (slot < (uint32_t)MQCAP) {
                                        sm.mq[par][m][slot] = key;
                                        taken |= bit;
                                    } else {
                                        ovf = true;
                                    }
                                }
                            }
                        }
                    }
                }
                sm.taken[tid] = taken;
                if (ovf) atomicOr(&sm.movf[par], 1u);
            }
        };
        // Wave w merges the queued mirror candidates of rows 16w..16w+15 of tile rt.
        auto mirror_merge = [&](int rt, bool refresh) __attribute__((always_inline)) {
            const int par = rt & 1;
            uint32_t mc = lane < QG_TR ? *(volatile uint32_t *)&sm.mcnt[par][lane] : 0u;
            u64 pend = __ballot(mc > 0) & (0xffffull << (16 * w));
            // Nothing queued for this wave's rows (nine tiles in ten at n = 2^20): leave before
            // the fence below, which would wait for the staging loads the step has just issued.
            if (pend == 0) return;
            merge_pending(
                pend, a.kcap, a.k, lane,
                [&](int m, u64 *&L, const u64 *&cq, int &nc) {
                    L = a.lists + (rrow0 + (int64_t)rt * QG_TR + m) * a.kcap;
                    cq = &sm.mq[par][m][0];
                    nc = min((int)__shfl(mc, m, 64), MQCAP);
                },
                [&](int m, u64 nt) {
                    if (lane == 0) {
                        sm.mcnt[par][m] = 0;
                        if (refresh) {
                            sm.mtau[par][m] = nt;
                            sm.T[par][m] = mirror_T(nt, sm.c[par][m], cmax, abound);
                        }
                    }
                });
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        };
        // Called by every wave after the barrier that ends tile rt.  Common case: each wave
        // merges its own rows, no further synchronisation (the rows' new thresholds are read
        // from the lists when the rows are visited again).  After an overflow the tile is
        // re-scanned against refreshed thresholds until every candidate found a slot; that
        // path is workgroup-uniform and uses barriers.
        auto mirror_service = [&](int rt) __attribute__((always_inline)) {
            const int par = rt & 1;
            if (*(volatile uint32_t *)&sm.movf[par] == 0) {
                mirror_merge(rt, false);
                return;
            }
            while (true) {
                mirror_merge(rt, true);
                __syncthreads();
                const uint32_t ovf = *(volatile uint32_t *)&sm.movf[par];
                __syncthreads();
                if (!ovf) break;
                if (tid == 0) sm.movf[par] = 0;
                __syncthreads();
                mirror_scan(rt, false);
                __syncthreads();
            }
        };

        int buf = 0;
        auto step = [&](auto kc_tag, int rt) __attribute__((always_inline)) {
            constexpr int kc = decltype(kc_tag)::value;
            constexpr bool last = kc == NK - 1;
            const bool more = !last || rt + 1 < n_rt;
            if (more) issue(last ? rt + 1 : rt, last ? 0 : kc + 1, buf ^ 1);
            __builtin_amdgcn_sched_barrier(0);
            if (kc == 0) {
                if (!diag && rt > 0) mirror_service(rt - 1);
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) {
                    f32x4 c0 = *(const f32x4 *)&sm.c[rt & 1][gg * 8 + h * 4];
                    f32x4 c1 = *(const f32x4 *)&sm.c[rt & 1][32 + gg * 8 + h * 4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        acc0[4 * gg + e] = c0[e];
                        acc1[4 * gg + e] = c1[e];
                    }
                }
            }
            const float *rb = &sm.r[buf][0];
            if constexpr (SPLIT) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int uh = ((2 * s + h) ^ sw) << 2, ul = ((4 + 2 * s + h) ^ sw) << 2;
                    const bf16x8 rh0 = __builtin_bit_cast(bf16x8, *(const f32x4 *)(rb + rbase0 + uh));
                    const bf16x8 rh1 = __builtin_bit_cast(bf16x8, *(const f32x4 *)(rb + rbase1 + uh));
                    const bf16x8 xh = __builtin_bit_cast(bf16x8, qreg[kc * QG_NSLAB + s]);
                    const bf16x8 xl = __builtin_bit_cast(bf16x8, qreg[kc * QG_NSLAB + 2 + s]);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rh0, xh, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rh1, xh, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rh0, xl, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rh1, xl, acc1, 0, 0, 0);
                    const bf16x8 rl0 = __builtin_bit_cast(bf16x8, *(const f32x4 *)(rb + rbase0 + ul));
                    const bf16x8 rl1 = __builtin_bit_cast(bf16x8, *(const f32x4 *)(rb + rbase1 + ul));
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rl0, xh, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rl1, xh, acc1, 0, 0, 0);
                }
            } else {
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
            }
            if (last) {
                // The epilogue is short vector work; at raised priority it does not queue behind
                // the matrix instructions of the other workgroup's wave on this SIMD, and the
                // wave is back to feeding the matrix pipe sooner (measured: -1.3 %).
                __builtin_amdgcn_s_setprio(1);
                float m2 = fminf(min16(acc0), min16(acc1));
                if (__ballot(m2 <= sm.tp[tid])) {
                    SelState st = load_state();
                    f32x16 blocks[2] = {acc0, acc1};
                    select_rare<2, QCAP>(blocks, (int32_t)(rrow0 + (int64_t)rt * QG_TR) + 4 * h, a.n,
                                         a.kcap, a.k, st, lane);
                    save_state(st);
                }
                if (!diag) mirror_scan(rt, true);
                __builtin_amdgcn_s_setprio(0);
            }
            if (more) stash(last ? 0 : kc + 1, (rt + 1) & 1);
            __syncthreads();
            buf ^= 1;
        };
        for (int rt = 0; rt < n_rt; ++rt) for_each_step<NK>(step, rt);
        {
            SelState st = load_state();
            merge_queues<QCAP>(st, a.kcap, a.k, lane);
        }
        if (!diag) mirror_service(n_rt - 1);
        __syncthreads();
    }
}

}  // namespace knn

#endif
