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

#include "knn_device.h"

namespace knn {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

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
        float s = 0.f;
        for (int c = lane; c < a.d; c += 64) {
            float v = x[c];
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
            for (int c = lane; c < a.dpad; c += 64) o[c] = c < a.d ? qscale * x[c] : 0.f;
        }
        if (a.r_out) {
            float *o = a.r_out + row * (int64_t)a.dpad;
            for (int c = lane; c < a.dpad; c += 64) o[c] = c < a.d ? rscale * x[c] : 0.f;
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
    u64 e0 = lane < kcap ? L[lane] : KEY_INF;
    u64 e1 = lane + 64 < kcap ? L[lane + 64] : KEY_INF;
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
    u64 tau_key = qvalid ? KEY_INF : 0ull;
    float tau_p = qvalid ? __builtin_inff() : -__builtin_inff();
    const int32_t selfj = (a.self_offset >= 0 && qvalid) ? (int32_t)(a.self_offset + myq) : -1;

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

    auto issue = [&](int rt, int kc) {
#pragma unroll
        for (int i = 0; i < NPASS; ++i) {
            gq[i] = *(const f32x4 *)(qsrc[i] + kc * DC);
            int64_t row = min((int64_t)rt * TR + lrow + i * ROWS_PER_PASS, a.nr - 1);
            gr[i] = *(const f32x4 *)(a.Rp + row * a.ldr + lcol + kc * DC);
        }
        if (kc == 0 && tid < TR) gc = a.cR[(int64_t)rt * TR + tid];
    };
    auto stash = [&](int buf, int kc) {
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
            float m4 = min16(acc[0]);
            m4 = fminf(m4, min16(acc[1]));
            m4 = fminf(m4, min16(acc[2]));
            m4 = fminf(m4, min16(acc[3]));
            if (__ballot(m4 <= tau_p)) {
                // Rare path, kept small on purpose: one 32x32 block at a time, its
                // 16 registers walked with a run-time index.
#pragma unroll 1
                for (int t = 0; t < 4; ++t) {
                    f32x16 v = t == 0 ? acc[0] : t == 1 ? acc[1] : t == 2 ? acc[2] : acc[3];
                    if (__ballot(min16(v) <= tau_p) == 0) continue;
                    const int32_t jbase = rt * TR + t * 32 + 4 * h;
                    bool again;
                    do {
                        bool ovf = false;
#pragma unroll 1
                        for (int r = 0; r < 16; ++r) {
                            float p = v[r];
                            bool c = p <= tau_p;
                            if (__ballot(c)) {
                                int32_t j = jbase + 8 * (r >> 2) + (r & 3);
                                u64 key = make_key(p, j);
                                if (c && key < tau_key && j < a.nr && j != selfj) {
                                    uint32_t slot = atomicAdd(&sm.cnt[w][ql], 1u);
                                    if (slot < (uint32_t)QCAP) {
                                        sm.cq[w][ql][slot] = key;
                                        p = __builtin_inff();     // taken: a re-scan must not see it again
                                    } else {
                                        ovf = true;
                                    }
                                }
                                v[r] = p;
                            }
                        }
                        again = __ballot(ovf) != 0;
                        // merge every non-empty queue of this wave into its list
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
                        uint32_t mycnt = *(volatile uint32_t *)&sm.cnt[w][ql];
                        u64 pend = __ballot(mycnt > 0) & 0xffffffffull;
                        while (pend) {
                            int qi = __builtin_ctzll(pend);
                            pend &= pend - 1;
                            int nc = min((int)__builtin_amdgcn_readlane(mycnt, qi), QCAP);
                            u64 nt = merge_one(Lw + (int64_t)qi * a.kcap, a.kcap, a.k, &sm.cq[w][qi][0], nc, lane);
                            if (ql == qi) {
                                tau_key = nt;
                                tau_p = nt == KEY_INF ? __builtin_inff() : ord2f((uint32_t)(nt >> 32));
                            }
                        }
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
                        if (lane < 32) sm.cnt[w][lane] = 0;
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
                    } while (again);
                }
            }
        }

        if (more) stash(buf ^ 1, nkc);
        __syncthreads();
        rt = nrt;
        kc = nkc;
    }
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

    if (a.mode == FIN_RESCORE_SQ || a.mode == FIN_RESCORE_COS) {
        // The k winners are priced again from the original rows, accumulating in
        // double: a direct sum of squared differences (or 1 - cos from the three
        // sums), so the reported value carries neither the cancellation of
        // |u|^2+|v|^2-2u.v nor that of 1-cos in fp32.  n*k*d work, HBM bound.
        const float *x = a.Q + q * (int64_t)a.d;
        const bool cosine = a.mode == FIN_RESCORE_COS;
        for (int r = 0; r < a.k; ++r) {
            int32_t j = (int32_t)(uint32_t)keys[r];
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
                            double t = ud - vd;
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
                        double t = ud - vd;
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
    } else {
        const float add = a.mode == FIN_ADD_SQ ? a.sq[q] : 1.0f;
        for (int r = lane; r < a.k; r += 64) {
            u64 key = keys[r];
            float p = ord2f((uint32_t)(key >> 32));
            float dist = fmaxf(p + add, 0.f);
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

hipError_t launch_finalize(const FinArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(finalize_rows, dim3((unsigned)a.nq), dim3(64), 0, stream, a);
    return hipGetLastError();
}

}  // namespace knn
