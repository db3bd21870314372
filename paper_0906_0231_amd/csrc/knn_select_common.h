// Shared device code of the selection: packed (distance, index) keys, wave helpers, the rank
// merge of candidate queues into sorted lists, and the rare path that walks a block of
// accumulators (paper Sect. 6: test against the current k-th smallest, keep the few survivors).
// Included by knn_kernels.hip only.
#ifndef KNN_SELECT_COMMON_H_
#define KNN_SELECT_COMMON_H_

namespace knn {

// ---------------------------------------------------------------------------
// keys: (distance, index) packed so that unsigned 64-bit order == (dist, idx) order
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t f2ord(float f)
{
    uint32_t u = __float_as_uint(f);
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float ord2f(uint32_t o)
{
    uint32_t u = (o & 0x80000000u) ? (o ^ 0x80000000u) : ~o;
    return __uint_as_float(u);
}
__device__ __forceinline__ u64 make_key(float p, int32_t j)
{
    // p + 0 turns -0 into +0: the two are the same distance and must tie (lower index first)
    return ((u64)f2ord(p + 0.f) << 32) | (u64)(uint32_t)j;
}
__device__ __forceinline__ u64 readlane64(u64 v, int src)
{
    uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, src);
    uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(v >> 32), src);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}


__device__ __forceinline__ float min16(const f32x16 &v)
{
    float m = fminf(v[0], v[1]);
#pragma unroll
    for (int r = 2; r < 16; ++r) m = fminf(m, v[r]);
    return m;
}

// Merge the nc queued candidates of one query into its sorted list L[0..kcap)
// (only the first k entries are live).  Whole wave; returns the new k-th key.
__device__ __forceinline__ u64 merge_one(u64 *L, int kcap, int k, const u64 *cq, int nc, int lane)
{
    // device-scope loads: the list may have been written by another wave of this CU since
    // this wave last looked at the same cache line; take it from the L2, not the vector L1
    u64 e0 = lane < kcap ? __hip_atomic_load(&L[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : KEY_INF;
    u64 e1 = lane + 64 < kcap ? __hip_atomic_load(&L[lane + 64], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                              : KEY_INF;
    u64 cm = lane < nc ? cq[lane] : KEY_INF;
    int inc0 = 0, inc1 = 0, crank = 0, cbase = 0;
    for (int i = 0; i < nc; ++i) {
        u64 ci = cq[i];                                   // same address in every lane
        inc0 += ci < e0;
        inc1 += ci < e1;
        int below = __popcll(__ballot(e0 < ci)) + __popcll(__ballot(e1 < ci));
        if (lane == i) cbase = below;
        crank += ci < cm;
    }
    int p0 = lane + inc0, p1 = lane + 64 + inc1, pc = cbase + crank;
    bool w0 = lane < kcap && p0 < k, w1 = lane + 64 < kcap && p1 < k, wc = lane < nc && pc < k;
    if (w0) L[p0] = e0;
    if (w1) L[p1] = e1;
    if (wc) L[pc] = cm;
    u64 tk = KEY_INF;
    bool has = false;
    if (w0 && p0 == k - 1) { tk = e0; has = true; }
    if (w1 && p1 == k - 1) { tk = e1; has = true; }
    if (wc && pc == k - 1) { tk = cm; has = true; }
    u64 m = __ballot(has);
    int src = m ? __builtin_ctzll(m) : 0;
    return readlane64(tk, src);
}

__device__ __forceinline__ u64 shfl64(u64 v, int src)
{
    uint32_t lo = __shfl((uint32_t)v, src, 64);
    uint32_t hi = __shfl((uint32_t)(v >> 32), src, 64);
    return ((u64)hi << 32) | lo;
}

// Several merges at once: the wave is cut into groups of gsz = kcap lanes (kcap <= 64) and
// every group rank-merges one queue into one list, exactly as merge_one does with the
// whole wave.  A merge is a dependent chain load -> rank -> store of L2 latency, so doing
// 64/kcap of them per round trip is what makes the rare path cheap for small k.
//   L, cq, nc: per lane, already those of the lane's group (L == nullptr: group idle).
// Returns, per lane, the new k-th key of its group's list (KEY_INF while not full).
__device__ __forceinline__ u64 merge_multi(u64 *L, const u64 *cq, int nc, int gsz, int k, int lane)
{
    const int e = lane & (gsz - 1);
    const int gbase = lane - e;
    const u64 gmask = (gsz >= 64 ? ~0ull : ((1ull << gsz) - 1ull)) << gbase;
    const bool act = L != nullptr;
    u64 e0 = act ? __hip_atomic_load(&L[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : KEY_INF;
    u64 cm = (act && e < nc) ? cq[e] : KEY_INF;
    int inc0 = 0, crank = 0, cbase = 0;
    for (int i = 0; __ballot(act && i < nc); ++i) {
        const bool live = act && i < nc;
        u64 ci = live ? cq[i] : KEY_INF;                // one address per group
        inc0 += live && ci < e0;
        int below = __popcll(__ballot(live && e0 < ci) & gmask);
        if (e == i) cbase = below;
        crank += live && ci < cm;
    }
    const int p0 = e + inc0, pc = cbase + crank;
    const bool w0 = act && p0 < k, wc = act && e < nc && pc < k;
    if (w0) L[p0] = e0;
    if (wc) L[pc] = cm;
    u64 tk = KEY_INF;
    bool has = false;
    if (w0 && p0 == k - 1) { tk = e0; has = true; }
    if (wc && pc == k - 1) { tk = cm; has = true; }
    u64 m = __ballot(has) & gmask;
    return shfl64(tk, m ? __builtin_ctzll(m) : lane);
}

// Merge every queue named by a bit of `pend` (bit i = item i, i < 64).  get(i, L, cq, nc)
// resolves an item to its list, queue and fill count; done(i, key) receives the list's new
// k-th key.  Items are taken 64/kcap at a time (one per lane group) when kcap <= 64.
template <typename Get, typename Done>
__device__ __forceinline__ void merge_pending(u64 pend, int kcap, int k, int lane, Get get, Done done)
{
    if (kcap > 64) {
        while (pend) {
            int i = __builtin_ctzll(pend);
            pend &= pend - 1;
            u64 *L;
            const u64 *cq;
            int nc;
            get(i, L, cq, nc);
            done(i, merge_one(L, kcap, k, cq, nc, lane));
        }
        return;
    }
    const int G = 64 / kcap;                            // 1, 2 or 4 groups
    const int gi = lane / kcap;
    while (pend) {
        int item[4] = {-1, -1, -1, -1};
#pragma unroll
        for (int g = 0; g < 4; ++g)
            if (g < G && pend) {
                item[g] = __builtin_ctzll(pend);
                pend &= pend - 1;
            }
        int mine = item[0];
#pragma unroll
        for (int g = 1; g < 4; ++g)
            if (gi == g) mine = item[g];
        // get() may shuffle: every lane calls it (idle groups with item 0, then discarded)
        u64 *L;
        const u64 *cq;
        int nc;
        get(mine >= 0 ? mine : 0, L, cq, nc);
        if (mine < 0) {
            L = nullptr;
            nc = 0;
        }
        u64 nt = merge_multi(L, cq, nc, kcap, k, lane);
#pragma unroll
        for (int g = 0; g < 4; ++g)
            if (g < G && item[g] >= 0) done(item[g], readlane64(nt, g * kcap));
    }
}

// State a wave keeps for the selection of its queries (32 or 64, see merge_queues).
struct SelState {
    u64 tau_key;      // current k-th best (distance, index) key of the lane's query; KEY_INF if fewer than k
    float tau_p;      // its distance part (+inf while the list is not full)
    int32_t selfj;    // reference index that is the lane's query itself, or -1
    u64 *Lw;          // the wave's 32 lists in global memory, kcap entries each
    u64 *cq;          // the wave's candidate queues in LDS: [32][QCAP]
    uint32_t *cnt;    // their fill counts: [32]
    uint32_t mine;    // QPW == 64 only: fill count of the lane's own queue (no other lane appends to it)
};

// Rank-merge candidate queues of this wave into their lists and refresh the thresholds.
// Whole wave.  Only queues holding at least min_fill candidates are merged, and those whose
// list is still short of k entries (no threshold yet): a merge costs about the same for one
// candidate as for QC, so the others wait -- their thresholds are merely stale, i.e. looser,
// until they fill up or the caller flushes with min_fill = 1.
// QPW: queries per wave -- 32 in the matrix kernels (lanes l and l+32 share query l%32),
// 64 in the fold kernel (one query per lane).
template <int QC, int QPW = 32>
__device__ __forceinline__ void merge_queues(SelState &st, int kcap, int k, int lane, uint32_t min_fill = 1)
{
    const int ql = lane & (QPW - 1);
    uint32_t mycnt;
    if (QPW == 64) {                               // one lane per queue: the count lives in a register
        mycnt = st.mine;
    } else {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        mycnt = *(volatile uint32_t *)&st.cnt[ql];
    }
    const bool due = mycnt >= min_fill || (mycnt > 0 && st.tau_key == KEY_INF);
    const u64 pend = __ballot(due) & (QPW == 64 ? ~0ull : 0xffffffffull);
    if (pend == 0) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // the queue entries written by other lanes
    merge_pending(
        pend, kcap, k, lane,
        [&](int qi, u64 *&L, const u64 *&cq, int &nc) {
            L = st.Lw + (int64_t)qi * kcap;
            cq = st.cq + qi * QC;
            nc = min((int)__shfl(mycnt, qi, 64), QC);
        },
        [&](int qi, u64 nt) {
            if (ql == qi && nt < st.tau_key) st.tau_key = nt;
        });
    st.tau_p = st.tau_key == KEY_INF ? __builtin_inff() : ord2f((uint32_t)(st.tau_key >> 32));
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    if (QPW == 64) {
        if (due) st.mine = 0;
    } else if (lane < 32) {
        if ((pend >> lane) & 1ull) st.cnt[lane] = 0;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
}

// The rare path of the selection: some accumulator of this wave is below its query's
// threshold.  One block of 16 registers at a time.  Every lane first marks, in a bit mask, which
// of its 16 values pass the threshold (constant register indices); then the wave loops while any
// lane has a bit left, each lane taking ITS lowest marked register -- different registers in
// different lanes in the same pass -- so the passes number as many as the busiest lane has
// candidates (one or two), not 16.  A survivor is tested exactly on the packed
// (distance, index) key, with the query itself and padding rows excluded, and appended to the
// query's queue in LDS.  Queues are merged into the lists lazily: when one is three quarters
// full, when a list is still short of k entries (no threshold yet), or when the caller flushes
// at the end of its sweep; until then the threshold is merely stale, i.e. looser, which only
// lets more candidates into the queue.  A full queue loses nothing: the lane keeps its bit,
// the queues are merged, and the lane tries again in the next pass.
//   jb0: reference row of register 0 of block 0 for this lane (tile base + 4*(lane/32));
//   block t adds 32t.  With QPW == 64 (fold kernel: one query per lane, registers are
//   consecutive references) register r of block t is row jb0 + 16t + r.
template <int NB, int QC, int QPW = 32>
__device__ __forceinline__ void select_rare(const f32x16 (&acc)[NB], int32_t jb0, int64_t nr, int kcap,
                                            int k, SelState &st, int lane)
{
    const int ql = lane & (QPW - 1);
#pragma unroll 1
    for (int t = 0; t < NB; ++t) {
        // the block, picked element by element with constant indices so that everything stays in
        // registers (a run-time index would give the array a home in scratch memory)
        f32x16 v;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float x = acc[0][e];
#pragma unroll
            for (int b = 1; b < NB; ++b) x = t == b ? acc[b][e] : x;
            v[e] = x;
        }
        uint32_t mask = 0;
#pragma unroll
        for (int e = 0; e < 16; ++e) mask |= v[e] <= st.tau_p ? 1u << e : 0u;
        if (__ballot(mask != 0) == 0) continue;
        const int32_t jbase = jb0 + t * (QPW == 64 ? 16 : 32);
        bool urgent = false;
        // every pass clears a bit in each busy lane, or merges the queue that was full: at most
        // 16 + 16 passes; the bound is a guard, not a mechanism
#pragma unroll 1
        for (int pass = 0; pass < 64 && __ballot(mask != 0); ++pass) {
            const int r = mask ? __builtin_ctz(mask) : 0;
            float p = v[0];
#pragma unroll
            for (int e = 1; e < 16; ++e) p = r == e ? v[e] : p;
            const int32_t j = QPW == 64 ? jbase + r : jbase + 8 * (r >> 2) + (r & 3);
            const u64 key = make_key(p, j);
            // the thresholds may have moved since the mask was made
            const bool want = mask != 0 && p <= st.tau_p && key < st.tau_key && j < nr && j != st.selfj;
            bool full = false;
            if (want) {
                uint32_t slot = QPW == 64 ? st.mine : atomicAdd(&st.cnt[ql], 1u);
                if (slot < (uint32_t)QC) {
                    st.cq[ql * QC + slot] = key;
                    if (QPW == 64) st.mine = slot + 1;
                    urgent |= slot + 1 >= (uint32_t)(QC * 3 / 4) || st.tau_key == KEY_INF;
                } else {
                    full = true;
                }
            }
            if (!full) mask &= mask - 1;           // done with this register (taken or rejected)
            if (__ballot(full)) {
                merge_queues<QC, QPW>(st, kcap, k, lane, QC * 3 / 4);
                urgent = false;
            }
        }
        if (__ballot(urgent)) merge_queues<QC, QPW>(st, kcap, k, lane, QC * 3 / 4);
    }
}

}  // namespace knn

#endif
