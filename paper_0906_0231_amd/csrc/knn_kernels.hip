// Device code of the exact kNN library for MI355X (gfx950, wave64).
//
// Three kernels make up one call:
//   prep_rows      -- one pass over the input rows: squared norms and the scaled /
//                     padded copies the tile kernel reads          (HBM bound)
//   knn_tiles      -- the fused kernel: distance tiles on the fp32 matrix cores,
//                     threshold test and k-best update in the epilogue; the
//                     distance matrix of the paper's Phase 1 (Sect. 5) is never
//                     written out, its Phase 2 (Sect. 6) runs on the accumulators
//   finalize_rows  -- merge of partial lists, optional re-score, final order
//
// Distances are evaluated in the expanded form  p(q, j) = c_j + sum_c Q'[q][c] R'[j][c]:
//   squared Euclidean:  Q' = -2 Q, R' = R,      c_j = |r_j|^2;  delta = p + |q|^2
//   cosine:             Q' = -Q/|Q|, R' = R/|R|, c_j = 0;        delta = p + 1
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
typedef __attribute__((address_space(3))) void *lds_ptr;

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
    return ((u64)f2ord(p) << 32) | (u64)(uint32_t)j;
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

// ---------------------------------------------------------------------------
// prep_rows: one wave per row.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prep_rows(PrepArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;

    // rows past the end of the reference set never win: c = +inf
    if (a.c_out) {
        int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
        if (g < a.n_cpad - a.n) a.c_out[a.n + g] = __builtin_inff();
    }
    for (int64_t row = wave; row < a.n; row += nwaves) {
        const float *x = a.X + row * (int64_t)a.d;
        // Hellinger (metric 2): everything below sees y = sqrt(x); sum (sqrt u - sqrt v)^2 is
        // the squared Euclidean distance of the square-rooted rows
        const bool root = a.metric == 2;
        if (a.metric == 5) {
            // Kullback-Leibler: sum q ln(q/r) = sum q ln q - sum q ln r.  The first sum does
            // not depend on the reference (deferred, s_out); the second is an inner product
            // of q with ln r.  ln 0 is replaced by a large negative finite value so that a
            // zero query coordinate still contributes exactly 0 on the matrix cores.
            float s = 0.f;
            for (int c = lane; c < a.d; c += 64) s += x[c] > 0.f ? x[c] * logf(x[c]) : 0.f;
            s = wave_sum(s);
            if (a.q_out) {
                float *o = a.q_out + row * (int64_t)a.dpad;
                for (int c = lane; c < a.dpad; c += 64) o[c] = c < a.d ? -x[c] : 0.f;
            }
            if (a.r_out) {
                float *o = a.r_out + row * (int64_t)a.dpad;
                for (int c = lane; c < a.dpad; c += 64) o[c] = c < a.d ? fmaxf(logf(x[c]), -104.f) : 0.f;
            }
            if (lane == 0) {
                if (a.c_out) a.c_out[row] = 0.f;
                if (a.s_out) a.s_out[row] = s;
            }
            continue;
        }
        float s = 0.f;
        for (int c = lane; c < a.d; c += 64) {
            float v = root ? sqrtf(x[c]) : x[c];
            s = fmaf(v, v, s);
        }
        s = wave_sum(s);
        float qscale, rscale, cval;
        if (a.metric == 1) {
            float inv = s > 0.f ? 1.0f / sqrtf(s) : 0.f;
            qscale = -inv;
            rscale = inv;
            cval = 0.f;
        } else {
            qscale = -2.f;
            rscale = 1.f;
            cval = s;
        }
        if (a.q_out) {
            float *o = a.q_out + row * (int64_t)a.dpad;
            for (int c = lane; c < a.dpad; c += 64) o[c] = c < a.d ? qscale * (root ? sqrtf(x[c]) : x[c]) : 0.f;
        }
        if (a.r_out) {
            float *o = a.r_out + row * (int64_t)a.dpad;
            for (int c = lane; c < a.dpad; c += 64) o[c] = c < a.d ? rscale * (root ? sqrtf(x[c]) : x[c]) : 0.f;
        }
        if (lane == 0) {
            if (a.c_out) a.c_out[row] = cval;
            if (a.s_out) a.s_out[row] = s;
        }
    }
}

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
    u64 *shared_tau;  // LDS [32]: bound shared with the other waves serving the same queries, or null
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
        if (st.shared_tau) atomicMin(&st.shared_tau[lane], st.tau_key);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
}

// The rare path of the selection: some accumulator of this wave is below its query's
// threshold.  One 32x32 block at a time, its 16 registers are walked with a run-time
// index (small code, no extra register pressure in the hot loop).  A survivor is tested
// exactly on the packed (distance, index) key, with the query itself and padding rows
// excluded, and appended to the query's queue in LDS.  Queues are merged into the lists
// lazily: when one is three quarters full, when a list is still short of k entries (no threshold
// yet), or when the caller flushes at the end of its sweep; until then the threshold is
// merely stale, i.e. looser, which only lets more candidates into the queue.  A full
// queue loses nothing: the value stays in the block copy and the block is walked again
// after the merge.
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
        f32x16 v;
        if (QPW == 64) {
            // The fold kernel passes its live accumulators: pick the block element by element
            // with constant indices, so that they stay in registers (a run-time index would
            // give the whole array a home in scratch memory, written every tile).
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float x = acc[0][e];
#pragma unroll
                for (int b = 1; b < NB; ++b) x = t == b ? acc[b][e] : x;
                v[e] = x;
            }
        } else {
            // The matrix kernels pass a copy made on this rare path only.
            v = acc[0];
#pragma unroll
            for (int b = 1; b < NB; ++b)
                if (t == b) v = acc[b];
        }
        if (__ballot(min16(v) <= st.tau_p) == 0) continue;
        const int32_t jbase = jb0 + t * (QPW == 64 ? 16 : 32);
        bool again;
        int rounds = 0;                            // 16 entries, QC per round: a few rounds at most
        do {
            bool ovf = false, urgent = false;
#pragma unroll 1
            for (int r = 0; r < 16; ++r) {
                float p = v[r];
                bool c = p <= st.tau_p;
                if (__ballot(c)) {
                    int32_t j = QPW == 64 ? jbase + r : jbase + 8 * (r >> 2) + (r & 3);
                    u64 key = make_key(p, j);
                    if (c && key < st.tau_key && j < nr && j != st.selfj) {
                        uint32_t slot = QPW == 64 ? st.mine++ : atomicAdd(&st.cnt[ql], 1u);
                        if (slot < (uint32_t)QC) {
                            st.cq[ql * QC + slot] = key;
                            // taken: a re-walk must not see it again.  NaN, not +inf: while a list
                            // is short of k entries its threshold is +inf, and an entry that came
                            // round again as (+inf, j) would enter the list a second time; the rank
                            // merge assumes distinct keys
                            p = __builtin_nanf("");
                            urgent |= slot + 1 >= (uint32_t)(QC * 3 / 4) || st.tau_key == KEY_INF;
                        } else {
                            ovf = true;
                        }
                    }
                    v[r] = p;
                }
            }
            again = __ballot(ovf) != 0 && ++rounds < 16;
            if (again || __ballot(urgent)) merge_queues<QC, QPW>(st, kcap, k, lane, QC * 3 / 4);
        } while (again);
    }
}

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
    st.shared_tau = nullptr;
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

    auto issue = [&](int rt, int kc) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NPASS; ++i) {
            gq[i] = *(const f32x4 *)(qsrc[i] + kc * DC);
            int64_t row = min((int64_t)rt * TR + lrow + i * ROWS_PER_PASS, a.nr - 1);
            gr[i] = *(const f32x4 *)(a.Rp + row * a.ldr + lcol + kc * DC);
        }
        if (kc == 0 && tid < TR) gc = a.cR[(int64_t)rt * TR + tid];
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
        const bool more = it + 1 < total;
        if (more) issue(nrt, nkc);

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

        if (more) stash(buf ^ 1, nkc);
        __syncthreads();
        rt = nrt;
        kc = nkc;
    }
    merge_queues<QCAP>(st, a.kcap, a.k, lane);
}

// ---------------------------------------------------------------------------
// knn_tiles_qres: the fused kernel with the query tile stationary in LDS
// (d padded <= 256).
//
// The streaming kernel above re-reads its 128 x d query tile for every reference
// tile; with 64 workgroups per XCD those tiles do not fit the 4 MB L2 and evict the
// shared reference stream as well, so every tile load misses.  Here the scaled query
// tile is loaded into LDS once per sweep (128 rows x (d+4) floats <= 130 KB of the
// 160 KB) and only reference rows stream.  One workgroup of 8 waves per CU:
//   wave = (query group i of 32 queries) x (reference half g of 64 rows of the tile),
//   two 32x32 accumulator blocks per wave.
// The two halves are independent pipelines: each stages only its own 64 reference rows
// (own LDS buffers) and synchronises only its own 4 waves, through a counter in LDS, so
// that a half waiting for its slowest wave (or walking a rare path) leaves the matrix
// pipe of every SIMD to the wave of the other half.  s_barrier would couple all 8.
// Each wave keeps its own partial list per query (its half of every reference tile);
// the two halves share the tighter of their two thresholds through LDS.
// ---------------------------------------------------------------------------
constexpr int QR_QCAP = 4;
constexpr int QR_HALF = 64;                       // reference rows per half tile
constexpr int QR_RBUF = QR_HALF * DC;             // floats per staging buffer

// R staging layout: 64-byte rows, 16-byte units XOR-swizzled so that both the
// row-contiguous stores and the 16-rows-same-unit fragment reads are conflict free.
__device__ __forceinline__ int qr_swz(int row) { return ((row >> 1) & 3) ^ ((row >> 3) & 1); }

__device__ __forceinline__ void group_sync(uint32_t *bar, uint32_t target, int lane)
{
    // LDS operations of a wave complete in order, so once this wave's counter update is
    // performed its staging stores are visible.  No global-memory wait: loads issued for
    // later steps stay in flight.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    if (lane == 0) atomicAdd(bar, 1u);
    while (__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target)
        __builtin_amdgcn_s_sleep(1);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__global__ __launch_bounds__(512) void knn_tiles_qres(TileArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const int qstr = a.dpad + 4;                  // odd number of 16-byte units per row
    float *sQ = (float *)smem_raw;                // [128][qstr]
    float *sR = sQ + TQ * qstr;                   // [2 halves][2 buffers][QR_RBUF]
    float *sC = sR + 4 * QR_RBUF;                 // [2][2][64]
    u64 *sCq = (u64 *)(sC + 4 * QR_HALF);         // [8 waves][32][QR_QCAP]
    u64 *sTau = sCq + 8 * 32 * QR_QCAP;           // [4 query groups][32]
    uint32_t *sCnt = (uint32_t *)(sTau + 4 * 32); // [8][32]
    uint32_t *sBar = sCnt + 8 * 32;               // [2]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int g = w >> 2;                         // reference half
    const int qi = w & 3;                         // query group
    const int gt = tid & 255;                     // thread index inside the half
    const int h = lane >> 5;
    const int ql = lane & 31;

    const int qt = blockIdx.x / a.S;
    const int split = blockIdx.x - qt * a.S;
    const int64_t qbase = (int64_t)qt * TQ;
    const int rt0 = split * a.rt_per_split;
    const int rt1 = min(rt0 + a.rt_per_split, a.n_rtiles);
    const int nk = a.dpad / DC;

    u64 *Lw = a.lists + ((int64_t)(split * 2 + g) * a.nq_pad + qbase + 32 * qi) * a.kcap;
    for (int i = lane; i < 32 * a.kcap; i += 64) Lw[i] = KEY_INF;
    const int64_t myq = qbase + 32 * qi + ql;
    const bool qvalid = myq < a.nq;
    if (lane < 32) {
        sCnt[w * 32 + lane] = 0;
        if (g == 0) sTau[qi * 32 + lane] = qvalid ? KEY_INF : 0ull;
    }
    if (tid < 2) sBar[tid] = 0;

    SelState st;
    st.tau_key = qvalid ? KEY_INF : 0ull;
    st.tau_p = qvalid ? __builtin_inff() : -__builtin_inff();
    st.selfj = (a.self_offset >= 0 && qvalid) ? (int32_t)(a.self_offset + myq) : -1;
    st.Lw = Lw;
    st.cq = sCq + w * 32 * QR_QCAP;
    st.cnt = sCnt + w * 32;
    st.shared_tau = sTau + qi * 32;
    st.mine = 0;

    // query tile -> LDS, once
    {
        const int upr = a.dpad >> 2;              // 16-byte units per row
        for (int u = tid; u < TQ * upr; u += 512) {
            int row = u / upr, c4 = u - row * upr;
            int64_t grow = min(qbase + row, a.nq - 1);
            *(f32x4 *)&sQ[row * qstr + c4 * 4] = *(const f32x4 *)(a.Qp + grow * a.ldq + c4 * 4);
        }
    }
    __syncthreads();

    // staging of this half's 64 reference rows: thread -> (row, 16-byte unit)
    const int lrow = gt >> 2, lunit = gt & 3;
    float *myR = sR + g * 2 * QR_RBUF;
    float *myC = sC + g * 2 * QR_HALF;
    uint32_t *myBar = sBar + g;
    const int st_off = lrow * DC + ((lunit ^ qr_swz(lrow)) << 2);
    f32x4 pre[2];
    float prec[2] = {0.f, 0.f};
    int irt = rt0, ikc = 0;                       // (tile, chunk) of the next load to issue

    auto issue = [&](int slot) {
        int64_t row = min((int64_t)irt * TR + g * QR_HALF + lrow, a.nr - 1);
        pre[slot] = *(const f32x4 *)(a.Rp + row * a.ldr + ikc * DC + lunit * 4);
        // every thread, every step: a fixed number of loads in flight lets the compiler
        // wait for exactly the older pair instead of draining the queue
        prec[slot] = a.cR[(int64_t)irt * TR + g * QR_HALF + (gt & (QR_HALF - 1))];
        if (++ikc == nk) { ikc = 0; ++irt; }
    };
    auto stash = [&](int slot, int buf, bool first_chunk) {
        *(f32x4 *)&myR[buf * QR_RBUF + st_off] = pre[slot];
        if (first_chunk && gt < QR_HALF) myC[buf * QR_HALF + gt] = prec[slot];
    };

    const int total = (rt1 - rt0) * nk;
    uint32_t epoch = 0;
    if (total > 0) {
        issue(0);
        if (total > 1) issue(1);
        stash(0, 0, true);
    }
    epoch += 4;
    group_sync(myBar, epoch, lane);

    f32x16 acc[2];
    const float *qp = sQ + (32 * qi + ql) * qstr + h * 4;
    // fragment read offsets of the two 32-row blocks of this half (swizzled units)
    int roff[2][NSLAB];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int s = 0; s < NSLAB; ++s) {
            int row = t * 32 + ql;
            roff[t][s] = row * DC + (((2 * s + h) ^ qr_swz(row)) << 2);
        }

    int rt = rt0, kc = 0;
    auto step = [&](int it, int slot) {
        // slot == it & 1: registers that held step `it` are free again, refill for it+2
        if (it + 2 < total) issue(slot);
        const int buf = it & 1;
        if (kc == 0) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) {
                    f32x4 cv = *(const f32x4 *)&myC[buf * QR_HALF + t * 32 + gg * 8 + h * 4];
                    acc[t][4 * gg + 0] = cv[0];
                    acc[t][4 * gg + 1] = cv[1];
                    acc[t][4 * gg + 2] = cv[2];
                    acc[t][4 * gg + 3] = cv[3];
                }
        }
        const float *rb = myR + buf * QR_RBUF;
        const float *qk = qp + kc * DC;
#pragma unroll
        for (int s = 0; s < NSLAB; ++s) {
            f32x4 qf = *(const f32x4 *)(qk + s * 8);
            f32x4 rf0 = *(const f32x4 *)(rb + roff[0][s]);
            f32x4 rf1 = *(const f32x4 *)(rb + roff[1][s]);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(rf0[c], qf[c], acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(rf1[c], qf[c], acc[1], 0, 0, 0);
            }
        }
        if (kc == nk - 1) {
            u64 sh = st.shared_tau[ql];            // the other half may have tightened the bound
            if (sh < st.tau_key) {
                st.tau_key = sh;
                st.tau_p = ord2f((uint32_t)(sh >> 32));
            }
            float m2 = fminf(min16(acc[0]), min16(acc[1]));
            if (__ballot(m2 <= st.tau_p)) {
                f32x16 blocks[2] = {acc[0], acc[1]};
                select_rare<2, QR_QCAP>(blocks, rt * TR + g * QR_HALF + 4 * h, a.nr, a.kcap, a.k, st, lane);
            }
        }
        int nkc = kc + 1, nrt = rt;
        if (nkc == nk) { nkc = 0; nrt = rt + 1; }
        if (it + 1 < total) stash(slot ^ 1, buf ^ 1, nkc == 0);
        epoch += 4;
        group_sync(myBar, epoch, lane);
        rt = nrt;
        kc = nkc;
    };
    for (int it = 0; it < total; it += 2) {
        step(it, 0);
        if (it + 1 < total) step(it + 1, 1);
    }
    merge_queues<QR_QCAP>(st, a.kcap, a.k, lane);
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

template <int DPAD>
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
    st.Lw = Lw;
    st.cq = &sm.cq[w][0][0];
    st.cnt = &sm.cnt[w][0];
    st.shared_tau = nullptr;
    st.mine = 0;

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
            if (__ballot(m2 <= st.tau_p)) {
                f32x16 blocks[2] = {acc0, acc1};
                select_rare<2, QCAP>(blocks, rt * QG_TR + 4 * h, a.nr, a.kcap, a.k, st, lane);
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
    uint32_t taken[256];                          // mirror entries of the current tile already queued
};

__device__ __forceinline__ float mirror_T(u64 tkey, float cj, float cmax, float abound)
{
    if (tkey == KEY_INF) return __builtin_inff();
    if (tkey == 0ull) return -__builtin_inff();   // row past the end: nothing may pass
    float t = ord2f((uint32_t)(tkey >> 32));
    float slack = (fabsf(t) + cmax + abound) * 3.814697265625e-06f;   // 2^-18
    return (t + cj) + slack + slack;
}

template <int DPAD>
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
            st.shared_tau = nullptr;
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
        // survivors, per-row queue (by tile parity).  Entries that found a slot are recorded
        // in a per-lane bit mask so that a re-scan after an overflow skips them (the
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
                            float p2 = (p - sm.c[par][m]) + cq;          // this pair seen from row m
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
        };
        // Wave w merges the queued mirror candidates of rows 16w..16w+15 of tile rt.
        auto mirror_merge = [&](int rt, bool refresh) __attribute__((always_inline)) {
            const int par = rt & 1;
            uint32_t mc = lane < QG_TR ? *(volatile uint32_t *)&sm.mcnt[par][lane] : 0u;
            u64 pend = __ballot(mc > 0) & (0xffffull << (16 * w));
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

// ---------------------------------------------------------------------------
// knn_fold<METRIC>: distances that are a fold over the coordinates but not an inner product
// (Sect. 3: a_{c+1} = dbar(u_c, v_c, a_c)); here dbar = a + |u - v| (Manhattan) and
// max(a, |u - v|) (Chebyshev).  This is the paper's own Phase 1 arithmetic (Sect. 5: every
// thread folds its pair's coordinates into a register), on the vector ALUs: two
// instructions per coordinate and pair (subtract; add or max with the |.| modifier), so
// the bound is the vector instruction rate, not the matrix rate.
//
// Lane = query (64 per wave, one accumulator per reference of a 32-row tile in its own
// registers, so the selection is the same register-axis test as in the matrix kernels).
// The reference coordinates are the same for all 64 lanes: they are read with scalar loads
// into scalar registers and enter the vector instructions as scalar operands -- no LDS, no
// vector registers, no barrier; the scalar cache shares them between the waves of a CU.
// For that the references are re-packed once, tile by tile, in the order the loop consumes
// them ([tile][4 coordinates][32 rows]): the scalar loads walk one pointer with constant
// offsets and need no address arithmetic per row.
// The query side uses the same packing with 64 rows per tile: a lane reads its query's four
// coordinates with one 16-byte load, the wave 1 KB contiguous, the slice of a wave is one
// contiguous block that is re-read per reference tile from the L2.  Waves are independent:
// each keeps 64 lists for its slice of the reference range.
//
// The slices of one query run at the same time and each starts with an empty list, i.e. no
// threshold.  A slice's k-th best distance is an upper bound of the final k-th best, so the
// slices publish theirs (atomic minimum on one word per query in global memory) and test
// against the smallest one published so far: a value above it cannot be among the final k.
// A stale read is merely a looser bound.  This keeps the number of queue insertions near
// that of an unsliced run instead of multiplying it by the number of slices.
// ---------------------------------------------------------------------------
constexpr int FOLD_NR = KNN_FOLD_NR;               // references per tile (accumulators per lane)
constexpr int FOLD_QCAP = 16;
#ifndef KNN_FOLD_WAVES
#define KNN_FOLD_WAVES 4
#endif
constexpr int FOLD_WAVES = KNN_FOLD_WAVES;          // waves (query groups) per workgroup

typedef const float __attribute__((address_space(4))) *const_f32_ptr;   // constant address space: scalar loads
typedef const f32x16 __attribute__((address_space(4))) *const_f32x16_ptr;

template <int METRIC>
__device__ __forceinline__ float fold_step(float u, float v, float acc)
{
    if (METRIC == 3) return acc + fabsf(u - v);
    return fmaxf(acc, fabsf(u - v));
}

template <int METRIC>
__global__ __launch_bounds__(64 * FOLD_WAVES) void knn_fold(FoldArgs a)
{
    __shared__ u64 s_cq[FOLD_WAVES][64][FOLD_QCAP];
    __shared__ uint32_t s_cnt[FOLD_WAVES][64];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    // The waves of a workgroup take consecutive query groups and the same slice of the
    // reference range: they read the same reference tiles at about the same time, so the
    // scalar cache fetches each 64-byte line once for all of them (its path to the L2 is narrow).
    // Workgroups are dealt to the 8 XCDs round-robin by number.  Renumber them so that an XCD
    // runs a contiguous range of (query block, slice) pairs: the slices of one query block then
    // run side by side on one XCD and its query values stay in that XCD's L2 between re-reads.
    // (The grid is a multiple of 8; numbers past the last pair fall out at the test below.)
    const uint32_t per_xcd = gridDim.x >> 3;
    const uint32_t vb = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    const int64_t qg = (int64_t)(vb / a.S) * FOLD_WAVES + w;
    const int split = vb % a.S;
    const int64_t q0 = qg * 64;
    if (q0 >= a.nq) return;                        // whole wave; the kernel has no barrier
    const int64_t myq = q0 + lane;                 // < nq_pad: the transposed copy is that wide
    const bool qvalid = myq < a.nq;

    u64 *Lw = a.lists + ((int64_t)split * a.nq_pad + q0) * a.kcap;
    for (int i = lane; i < 64 * a.kcap; i += 64) Lw[i] = KEY_INF;
    s_cnt[w][lane] = 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");

    SelState st;
    st.tau_key = qvalid ? KEY_INF : 0ull;
    st.tau_p = qvalid ? __builtin_inff() : -__builtin_inff();
    st.selfj = (a.self_offset >= 0 && qvalid) ? (int32_t)(a.self_offset + myq) : -1;
    st.Lw = Lw;
    st.cq = &s_cq[w][0][0];
    st.cnt = &s_cnt[w][0];
    st.shared_tau = nullptr;
    st.mine = 0;

    const int64_t j_begin = (int64_t)split * a.refs_per_split;
    const int64_t j_end = min(a.nr, j_begin + a.refs_per_split);
    const f32x4 *qp = (const f32x4 *)(a.Qpk + qg * (int64_t)(a.dpad >> 2) * 256) + lane;
    uint32_t *mybound = a.bound + myq;
    uint32_t published = 0xffffffffu;
    const_f32_ptr Rc = (const_f32_ptr)a.Rpk;       // never written while this kernel runs
    const int ncq = a.dpad >> 2;

    for (int64_t j0 = j_begin; j0 < j_end; j0 += FOLD_NR) {
        f32x16 acc[FOLD_NR / 16];                  // register 16 t + r: reference j0 + 16 t + r
        // what the other slices have reached; read now, used after the tile
        const uint32_t seen = __hip_atomic_load(mybound, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int t = 0; t < FOLD_NR / 16; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
        // rows past the end of the set are zero rows in the packed copy; the selection discards them
        const_f32x16_ptr tile = (const_f32x16_ptr)(Rc + (j0 / FOLD_NR) * (int64_t)ncq * (FOLD_NR * 4));
        f32x4 qn = qp[0];
        // The scalar loads run one batch (8 rows x 4 coordinates = 128 bytes) ahead of the vector
        // instructions that consume them; the batch after a tile's last one belongs to the next
        // tile (or to the padding behind the last tile) and is simply dropped.
        f32x16 cur0 = tile[0], cur1 = tile[1];
        for (int cq = 0; cq < ncq; ++cq) {
            const f32x4 q = qn;
            if (cq + 1 < ncq) qn = qp[(cq + 1) * 64];
#pragma unroll
            for (int b = 0; b < FOLD_NR / 8; ++b) {
                const f32x16 nxt0 = tile[(cq * (FOLD_NR / 8) + b + 1) * 2];
                const f32x16 nxt1 = tile[(cq * (FOLD_NR / 8) + b + 1) * 2 + 1];
                __builtin_amdgcn_sched_barrier(0);
                // coordinate outermost: consecutive instructions update different accumulators
#pragma unroll
                for (int e = 0; e < 4; ++e) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        acc[b >> 1][8 * (b & 1) + i] =
                            fold_step<METRIC>(q[e], cur0[4 * i + e], acc[b >> 1][8 * (b & 1) + i]);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        acc[b >> 1][8 * (b & 1) + 4 + i] =
                            fold_step<METRIC>(q[e], cur1[4 * i + e], acc[b >> 1][8 * (b & 1) + 4 + i]);
                }
                cur0 = nxt0;
                cur1 = nxt1;
            }
        }
        float m = min16(acc[0]);
#pragma unroll
        for (int t = 1; t < FOLD_NR / 16; ++t) m = fminf(m, min16(acc[t]));
        if (seen != 0xffffffffu) st.tau_p = fminf(st.tau_p, ord2f(seen));
        if (__ballot(m <= st.tau_p)) {
            select_rare<FOLD_NR / 16, FOLD_QCAP, 64>(acc, (int32_t)j0, a.nr, a.kcap, a.k, st, lane);
            const uint32_t mine = (uint32_t)(st.tau_key >> 32);
            if (qvalid && st.tau_key != KEY_INF && mine < published) {
                atomicMin(mybound, mine);
                published = mine;
            }
        }
    }
    merge_queues<FOLD_QCAP, 64>(st, a.kcap, a.k, lane);
}

// pack_tiles: Xpk[tile t][coordinate quad cq][row r][e] = X[T t + r][4 cq + e], zero outside
// (T = rows_per_tile).
// One thread per (row, quad); consecutive threads take consecutive quads of a row.
__global__ __launch_bounds__(256) void pack_tiles(PackArgs a)
{
    const int ncq = a.dpad >> 2;
    const int FOLD_NR = a.rows_per_tile;
    const int64_t total = (a.n + FOLD_NR - 1) / FOLD_NR * FOLD_NR * (int64_t)ncq;
    for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < total; g += (int64_t)gridDim.x * 256) {
        const int64_t row = g / ncq;
        const int cq = (int)(g - row * ncq);
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int c = 4 * cq + e;
            v[e] = (row < a.n && c < a.d) ? a.X[row * (int64_t)a.d + c] : 0.f;
        }
        const int64_t t = row / FOLD_NR;
        const int r = (int)(row - t * FOLD_NR);
        *(f32x4 *)(a.Xpk + ((t * ncq + cq) * FOLD_NR + r) * 4) = v;
        if (a.bound != nullptr && cq == 0 && row < a.n) a.bound[row] = 0xffffffffu;
    }
}

// ---------------------------------------------------------------------------
// select_rows: batched partial sort of a materialised matrix -- the paper's Phase 2 as it
// states it (Sect. 6): for every row of A[m, n], the k smallest entries.  Bound by HBM
// (4 bytes per element, read once); nothing else is moved.
//
// One wave per (row, column segment).  The paper gives a thread block a row, lets the
// threads stride it for coalescing, compares each element with the heap's top and
// buffers the few survivors per thread before a serialised push.  Here a lane reads 32
// consecutive-by-4 floats per iteration (eight 1 KB wave loads in flight), keeps their
// minimum, and the whole wave takes one branch on "any lane below the threshold"; the
// survivors are compacted into a wave queue in LDS with ballot/popcount and rank-merged
// into the row's sorted list (also in LDS) by the same code as the fused kernels.
// ---------------------------------------------------------------------------
constexpr int SEL_LOADS = 8;                      // float4 loads in flight per lane
constexpr int SEL_CHUNK = 64 * 4 * SEL_LOADS;     // columns per wave iteration

__global__ __launch_bounds__(256) void select_rows(SelectArgs a)
{
    __shared__ u64 sList[4][KNN_MAX_KCAP];
    __shared__ u64 sQueue[4][64];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int64_t gw = (int64_t)blockIdx.x * 4 + w;
    if (gw >= a.m * a.S) return;                  // whole wave; no barriers in this kernel
    const int64_t row = gw / a.S;
    const int seg = (int)(gw - row * a.S);
    const int64_t c0 = (int64_t)seg * a.seg;
    const int64_t c1 = min(c0 + a.seg, a.n);
    const float *Arow = a.A + row * a.lda;
    u64 *L = &sList[w][0];
    u64 *Q = &sQueue[w][0];
    for (int i = lane; i < a.kcap; i += 64) L[i] = KEY_INF;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");

    u64 tau_key = KEY_INF;
    float tau_p = __builtin_inff();
    int count = 0;                                // queued candidates (wave-uniform)
    const float INF = __builtin_inff();

    auto flush = [&]() __attribute__((always_inline)) {
        if (count == 0) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        u64 nt = merge_one(L, a.kcap, a.k, Q, count, lane);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        tau_key = nt;
        tau_p = nt == KEY_INF ? INF : ord2f((uint32_t)(nt >> 32));
        count = 0;
    };

    for (int64_t base = c0; base < c1; base += SEL_CHUNK) {
        f32x4 v[SEL_LOADS];
#pragma unroll
        for (int j = 0; j < SEL_LOADS; ++j) {
            const int64_t col = base + j * 256 + lane * 4;
            if (a.vec4 && col + 3 < c1) {
                v[j] = *(const f32x4 *)(Arow + col);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[j][e] = col + e < c1 ? Arow[col + e] : INF;
            }
        }
        float m = INF;
#pragma unroll
        for (int j = 0; j < SEL_LOADS; ++j) m = fminf(m, fminf(fminf(v[j][0], v[j][1]), fminf(v[j][2], v[j][3])));
        if (__ballot(m <= tau_p) == 0) continue;
        // rare path: element by element, survivors compacted into the wave queue
#pragma unroll
        for (int j = 0; j < SEL_LOADS; ++j) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float p = v[j][e];
                const bool c = p <= tau_p;
                if (__ballot(c)) {
                    const int64_t col = base + j * 256 + lane * 4 + e;
                    const u64 key = make_key(p, (int32_t)col);
                    const bool pass = c && key < tau_key && col < c1;
                    u64 bal = __ballot(pass);
                    int np = __popcll(bal);
                    if (np) {
                        if (count + np > 64) flush();     // thresholds move; entries already chosen stay valid candidates
                        int pos = count + __popcll(bal & ((1ull << lane) - 1ull));
                        if (pass) Q[pos] = key;
                        count += np;
                    }
                }
            }
        }
        if (count >= 32 || tau_key == KEY_INF) flush();
    }
    flush();
    u64 *out = a.lists + ((int64_t)seg * a.m + row) * a.kcap;
    for (int i = lane; i < a.kcap; i += 64) out[i] = L[i];
}

// ---------------------------------------------------------------------------
// finalize_rows: one wave per query.
// ---------------------------------------------------------------------------
constexpr int FIN_MAX = KNN_FIN_MAX;   // most keys one query can bring (S * kcap)

__device__ __forceinline__ void bitonic_sort_lds(u64 *keys, int n, int lane)
{
    for (int size = 2; size <= n; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = lane; i < (n >> 1); i += 64) {
                int lo = 2 * i - (i & (stride - 1));
                int hi = lo + stride;
                bool up = (lo & size) == 0;
                u64 x = keys[lo], y = keys[hi];
                if ((x > y) == up) {
                    keys[lo] = y;
                    keys[hi] = x;
                }
            }
            __syncthreads();
        }
    }
}

__global__ __launch_bounds__(64) void finalize_rows(FinArgs a)
{
    __shared__ u64 keys[FIN_MAX];
    __shared__ u64 outk[KNN_MAX_KCAP];
    const int lane = threadIdx.x;
    const int64_t q = blockIdx.x;

    const int nin = a.S * a.kcap;
    int npow = 1;
    while (npow < nin) npow <<= 1;
    for (int i = lane; i < npow; i += 64) {
        u64 v = KEY_INF;
        if (i < nin) {
            int s = i / a.kcap, e = i - s * a.kcap;
            v = a.lists[((int64_t)s * a.nq_pad + q) * a.kcap + e];
        }
        keys[i] = v;
    }
    __syncthreads();
    if (a.S > 1) bitonic_sort_lds(keys, npow, lane);

    int kpow = 1;
    while (kpow < a.k) kpow <<= 1;
    for (int i = lane; i < kpow; i += 64) outk[i] = KEY_INF;
    __syncthreads();

    if (a.mode == FIN_RESCORE_L1 || a.mode == FIN_RESCORE_LINF || a.mode == FIN_RESCORE_KL) {
        // the same re-pricing of the k winners in double for the distances of the fold family
        const float *x = a.Q + q * (int64_t)a.d;
        for (int r = 0; r < a.k; ++r) {
            int32_t j = (int32_t)(uint32_t)keys[r];
            if (j < 0 || j >= a.nr) {
                if (lane == 0) outk[r] = KEY_INF;
                continue;
            }
            const float *y = a.R + (int64_t)j * a.d;
            double s = 0.0;
            for (int c = lane; c < a.d; c += 64) {
                double ud = (double)x[c], vd = (double)y[c];
                if (a.mode == FIN_RESCORE_L1) s += fabs(ud - vd);
                else if (a.mode == FIN_RESCORE_LINF) s = fmax(s, fabs(ud - vd));
                else if (ud > 0.0) s += ud * log(ud / vd);
            }
            if (a.mode == FIN_RESCORE_LINF) {
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) s = fmax(s, __shfl_xor(s, o, 64));
            } else {
                s = wave_sum_f64(s);
            }
            if (lane == 0) outk[r] = make_key((float)s, j);
        }
    } else if (a.mode == FIN_RESCORE_SQ || a.mode == FIN_RESCORE_COS || a.mode == FIN_RESCORE_HEL) {
        // The k winners are priced again from the original rows, accumulating in
        // double: a direct sum of squared differences (or 1 - cos from the three
        // sums), so the reported value carries neither the cancellation of
        // |u|^2+|v|^2-2u.v nor that of 1-cos in fp32.  n*k*d work, HBM bound.
        const float *x = a.Q + q * (int64_t)a.d;
        const bool cosine = a.mode == FIN_RESCORE_COS;
        const bool root = a.mode == FIN_RESCORE_HEL;
        for (int r = 0; r < a.k; ++r) {
            int32_t j = (int32_t)(uint32_t)keys[r];
            if (j < 0 || j >= a.nr) {             // an unfilled slot (cannot happen for k <= nr - self)
                if (lane == 0) outk[r] = KEY_INF;
                continue;
            }
            const float *y = a.R + (int64_t)j * a.d;
            double s = 0.0, uu = 0.0, vv = 0.0;
            if (a.vec4) {
                for (int c = lane * 4; c < a.d; c += 256) {
                    f32x4 u = *(const f32x4 *)(x + c), v = *(const f32x4 *)(y + c);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        double ud = (double)u[e], vd = (double)v[e];
                        if (cosine) {
                            s = fma(ud, vd, s);
                            uu = fma(ud, ud, uu);
                            vv = fma(vd, vd, vv);
                        } else {
                            double t = root ? sqrt(ud) - sqrt(vd) : ud - vd;
                            s = fma(t, t, s);
                        }
                    }
                }
            } else {
                for (int c = lane; c < a.d; c += 64) {
                    double ud = (double)x[c], vd = (double)y[c];
                    if (cosine) {
                        s = fma(ud, vd, s);
                        uu = fma(ud, ud, uu);
                        vv = fma(vd, vd, vv);
                    } else {
                        double t = root ? sqrt(ud) - sqrt(vd) : ud - vd;
                        s = fma(t, t, s);
                    }
                }
            }
            s = wave_sum_f64(s);
            if (cosine) {
                uu = wave_sum_f64(uu);
                vv = wave_sum_f64(vv);
                s = (uu == 0.0 || vv == 0.0) ? 1.0 : 1.0 - s / (sqrt(uu) * sqrt(vv));
                if (s < 0.0) s = 0.0;
            }
            if (lane == 0) outk[r] = make_key((float)s, j);
        }
    } else if (a.mode == FIN_SELECT) {
        for (int r = lane; r < a.k; r += 64) outk[r] = keys[r];   // keys are (value, column) already
    } else {
        const float add = a.mode == FIN_ADD_ONE ? 1.0f : a.sq[q];
        for (int r = lane; r < a.k; r += 64) {
            u64 key = keys[r];
            float p = ord2f((uint32_t)(key >> 32));
            float dist = a.mode == FIN_ADD_SQ_SIGNED ? p + add : fmaxf(p + add, 0.f);
            outk[r] = make_key(dist, (int32_t)(uint32_t)key);
        }
    }
    __syncthreads();
    bitonic_sort_lds(outk, kpow, lane);
    for (int r = lane; r < a.k; r += 64) {
        u64 key = outk[r];
        a.idx[q * a.k + r] = (int32_t)(uint32_t)key;
        a.dist[q * a.k + r] = ord2f((uint32_t)(key >> 32));
    }
}

// ---------------------------------------------------------------------------
// mfma_only: calibration.  Nothing but the contraction's matrix instruction on four
// independent accumulators per wave; no memory traffic inside the loop.  Timing it gives
// the fp32 matrix rate the device sustains under load (clock included).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mfma_only(int64_t groups_of_16, float *sink)
{
    f32x16 a0 = {}, a1 = {}, a2 = {}, a3 = {};
    // operands with busy mantissas that differ from lane to lane and from one instruction to
    // the next, as real data do (constant operands would flatter the power draw); products
    // of both signs keep the sums bounded
    float x[4], y[4];
    uint32_t hsh = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        hsh = hsh * 1664525u + 1013904223u;
        x[u] = __uint_as_float(0x3f000000u | (hsh >> 9)) * ((hsh & 256u) ? 1.f : -1.f);
        hsh = hsh * 1664525u + 1013904223u;
        y[u] = __uint_as_float(0x3f000000u | (hsh >> 9)) * ((hsh & 256u) ? 1.f : -1.f) * 9.5367431640625e-07f;
    }
    for (int64_t i = 0; i < groups_of_16; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a0 = __builtin_amdgcn_mfma_f32_32x32x2f32(x[u], y[u], a0, 0, 0, 0);
            a1 = __builtin_amdgcn_mfma_f32_32x32x2f32(x[(u + 1) & 3], y[u], a1, 0, 0, 0);
            a2 = __builtin_amdgcn_mfma_f32_32x32x2f32(x[(u + 2) & 3], y[(u + 1) & 3], a2, 0, 0, 0);
            a3 = __builtin_amdgcn_mfma_f32_32x32x2f32(x[(u + 3) & 3], y[(u + 2) & 3], a3, 0, 0, 0);
        }
    }
    float t = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) t += (a0[e] + a1[e]) + (a2[e] + a3[e]);
    sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = t;
}

// valu_only: the fold kernel's instruction pair and nothing else: 32 independent chains, the
// subtrahend a scalar register, 128 distinct (query value, scalar) combinations per pass.
__global__ __launch_bounds__(256) void valu_only(int64_t groups_of_128, const float *seed, float *sink)
{
    float acc[32];
#pragma unroll
    for (int r = 0; r < 32; ++r) acc[r] = 0.f;
    float q[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = (float)((threadIdx.x & 63) + 64 * i) * 0.001f;
    float sv[16];                                  // wave-uniform, from memory: scalar registers
#pragma unroll
    for (int i = 0; i < 16; ++i) sv[i] = seed[i];
    for (int64_t it = 0; it < groups_of_128; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(q[i]));   // opaque: nothing is hoisted or merged
        // consecutive instructions belong to different chains, as in knn_fold
#pragma unroll
        for (int g = 0; g < 8; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[4 * g + i] += fabsf(q[g] - sv[i * 4 + e]);
    }
    float t = 0.f;
#pragma unroll
    for (int r = 0; r < 32; ++r) t += acc[r];
    sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = t;
}

hipError_t launch_valu_calibration(int64_t pairs_per_wave, int blocks, int waves_per_simd, float *sink, hipStream_t stream)
{
    // the seed values live at the end of the sink, past the part the kernel writes
    const float *seed = sink + (int64_t)blocks * 256;
    hipLaunchKernelGGL(valu_only, dim3((unsigned)blocks), dim3(256), 0, stream, pairs_per_wave / 128, seed, sink);
    (void)waves_per_simd;
    return hipGetLastError();
}

hipError_t launch_mfma_calibration(int64_t mfma_per_wave, int blocks, float *sink, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_only, dim3((unsigned)blocks), dim3(256), 0, stream, mfma_per_wave / 16, sink);
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

hipError_t launch_tiles(const TileArgs &a, hipStream_t stream)
{
    int64_t blocks = (int64_t)a.n_qtiles * a.S;
    hipLaunchKernelGGL(knn_tiles, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

size_t qres_lds_bytes(int dpad)
{
    return (size_t)TQ * (dpad + 4) * 4 + 4 * QR_RBUF * 4 + 4 * QR_HALF * 4 + 8 * 32 * QR_QCAP * 8 +
           4 * 32 * 8 + 8 * 32 * 4 + 16;
}

hipError_t launch_tiles_qres(const TileArgs &a, hipStream_t stream)
{
    static thread_local int configured_dev = -1;
    size_t lds = qres_lds_bytes(a.dpad);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (configured_dev != dev) {
        e = hipFuncSetAttribute((const void *)knn_tiles_qres, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)qres_lds_bytes(KNN_QRES_MAX_D));
        if (e != hipSuccess) return e;
        configured_dev = dev;
    }
    int64_t blocks = (int64_t)a.n_qtiles * a.S;
    hipLaunchKernelGGL(knn_tiles_qres, dim3((unsigned)blocks), dim3(512), lds, stream, a);
    return hipGetLastError();
}

hipError_t launch_tiles_qreg(const TileArgs &a, hipStream_t stream)
{
    int64_t blocks = (int64_t)a.n_qtiles * a.S;
    dim3 grid((unsigned)blocks), block(256);
    switch (a.dpad) {
    case 32: hipLaunchKernelGGL(knn_tiles_qreg<32>, grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL(knn_tiles_qreg<64>, grid, block, 0, stream, a); break;
    case 96: hipLaunchKernelGGL(knn_tiles_qreg<96>, grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL(knn_tiles_qreg<128>, grid, block, 0, stream, a); break;
    case 160: hipLaunchKernelGGL(knn_tiles_qreg<160>, grid, block, 0, stream, a); break;
    case 192: hipLaunchKernelGGL(knn_tiles_qreg<192>, grid, block, 0, stream, a); break;
    case 224: hipLaunchKernelGGL(knn_tiles_qreg<224>, grid, block, 0, stream, a); break;
    case 256: hipLaunchKernelGGL(knn_tiles_qreg<256>, grid, block, 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// largest c_j (squared norm) of the data set: scale of the mirror slack
__global__ __launch_bounds__(1024) void reduce_max(const float *c, int64_t n, float *out)
{
    __shared__ float part[16];
    float m = 0.f;
    for (int64_t i = threadIdx.x; i < n; i += 1024) m = fmaxf(m, c[i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < 16; ++i) m = fmaxf(m, part[i]);
        *out = m;
    }
}

hipError_t launch_reduce_max(const float *c, int64_t n, float *out, hipStream_t stream)
{
    hipLaunchKernelGGL(reduce_max, dim3(1), dim3(1024), 0, stream, c, n, out);
    return hipGetLastError();
}

hipError_t launch_pairs_qreg(const PairArgs &a, int blocks, hipStream_t stream)
{
    dim3 grid((unsigned)blocks), block(256);
    switch (a.dpad) {
    case 32: hipLaunchKernelGGL(knn_pairs_qreg<32>, grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL(knn_pairs_qreg<64>, grid, block, 0, stream, a); break;
    case 96: hipLaunchKernelGGL(knn_pairs_qreg<96>, grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL(knn_pairs_qreg<128>, grid, block, 0, stream, a); break;
    case 160: hipLaunchKernelGGL(knn_pairs_qreg<160>, grid, block, 0, stream, a); break;
    case 192: hipLaunchKernelGGL(knn_pairs_qreg<192>, grid, block, 0, stream, a); break;
    case 224: hipLaunchKernelGGL(knn_pairs_qreg<224>, grid, block, 0, stream, a); break;
    case 256: hipLaunchKernelGGL(knn_pairs_qreg<256>, grid, block, 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
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
    hipLaunchKernelGGL(select_rows, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_finalize(const FinArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(finalize_rows, dim3((unsigned)a.nq), dim3(64), 0, stream, a);
    return hipGetLastError();
}

}  // namespace knn
