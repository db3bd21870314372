// Distances that are coordinate folds but not inner products (paper Sect. 3) on the vector ALUs:
// pack_tiles, knn_fold; and the two calibration kernels.  Included by knn_kernels.hip only.
#ifndef KNN_FOLD_KERNELS_H_
#define KNN_FOLD_KERNELS_H_

namespace knn {

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

// (four waves per SIMD: the register allocation is capped at 128 so that the rare path cannot cost one)
template <int METRIC>
__global__ __attribute__((amdgpu_waves_per_eu(4, 4))) __launch_bounds__(64 * FOLD_WAVES) void knn_fold(FoldArgs a)
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

// ---------------------------------------------------------------------------
// knn_fold_dist<METRIC, MODE>: the fold of knn_fold with the paper's two phases kept apart
// (Sect. 5-6): the distances are written out, select_rows picks the k smallest per row
// afterwards.  With DIST_TRIANGLE (knn_build: these distances are symmetric, Sect. 3) a wave
// computes only the tiles from its own diagonal tile on and stores each value beyond it twice,
// D[q][j] and D[j][q] -- half the vector instructions, which are what bounds this path.
// DIST_RECT_MIRROR: two different row panels of one data set, every value stored twice, the
// mirrored one into the buffer of the transposed block (see knn_dist_qreg).
// Same loop as knn_fold: lane = query, one accumulator per reference of a 64-row tile, reference
// coordinates through scalar registers.  The waves of a workgroup take consecutive query groups
// and walk the same tiles together (the scalar cache fetches a line once for all of them); a
// wave skips the at most three tiles below its own diagonal.
// Stores: in the mirrored part the lanes hold 64 consecutive queries of one row (256 bytes per
// instruction); the direct part, where a lane holds 64 consecutive columns of ITS row, goes
// through a per-wave LDS buffer 16 columns at a time and leaves as 64-byte row segments.
// ---------------------------------------------------------------------------
constexpr int FD_PITCH = 20;                       // floats per row of the transposition buffer (16 + pad, 16-byte aligned)
constexpr int FB_PITCH = 20;                       // 16 chunk minima per row (+ pad, 16-byte aligned)
constexpr int FM_PITCH = 66;                       // the same buffer as 16 rows of 64 (+2) for the mirrored minima
static_assert(16 * FM_PITCH <= 64 * FD_PITCH, "the mirrored rows must fit the transposition buffer");

template <int METRIC, int MODE>
__global__ __attribute__((amdgpu_waves_per_eu(4, 4))) __launch_bounds__(64 * FOLD_WAVES) void knn_fold_dist(FoldDistArgs a)
{
    __shared__ __attribute__((aligned(16))) float s_tr[FOLD_WAVES][64 * FD_PITCH];
    __shared__ __attribute__((aligned(16))) float s_min[FOLD_WAVES][64 * FB_PITCH];   // chunk minima of 8 tiles per row
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    // chunk-major numbering, as in knn_dist_qreg: the 8 XCDs get equal shares of every chunk index
    const int chunk = blockIdx.x / a.n_qblocks;
    const int qb = blockIdx.x - chunk * a.n_qblocks;
    const int64_t qg = (int64_t)qb * FOLD_WAVES + w;
    const int64_t q0 = qg * 64;
    if (q0 >= a.nq) return;                        // whole wave; the kernel has no barrier
    const int64_t myq = q0 + lane;                 // < nq_pad: the matrix and the packed copy are that tall
    const int64_t selfj = a.self_offset >= 0 ? a.self_offset + myq : -1;

    // tiles of 64 references; the workgroup's first diagonal tile is that of its first wave
    constexpr bool TRI = MODE == DIST_TRIANGLE;
    const int64_t t_first = TRI ? (int64_t)qb * FOLD_WAVES : 0;
    // chunk boundaries do not depend on the query block (the workgroups of a chunk index walk
    // the same tiles together); chunks that end below the block's diagonal have nothing to do
    const int64_t t0 = max((int64_t)chunk * a.chunk, t_first);
    const int64_t t1 = min((int64_t)chunk * a.chunk + a.chunk, a.n_tiles);

    const f32x4 *qp = (const f32x4 *)(a.Qpk + qg * (int64_t)(a.dpad >> 2) * 256) + lane;
    const_f32_ptr Rc = (const_f32_ptr)a.Rpk;       // never written while this kernel runs
    const int ncq = a.dpad >> 2;
    float *tr = &s_tr[w][0];

    for (int64_t tj = t0; tj < t1; ++tj) {
        if (TRI && tj < qg) continue;              // below this wave's diagonal: the other wave's mirror writes it
        const int64_t j0 = tj * FOLD_NR;
        f32x16 acc[FOLD_NR / 16];                  // register 16 t + r: reference j0 + 16 t + r
#pragma unroll
        for (int t = 0; t < FOLD_NR / 16; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
        const_f32x16_ptr tile = (const_f32x16_ptr)(Rc + tj * (int64_t)ncq * (FOLD_NR * 4));
        f32x4 qn = qp[0];
        f32x16 cur0 = tile[0], cur1 = tile[1];     // scalar loads run one batch ahead, as in knn_fold
        for (int cq = 0; cq < ncq; ++cq) {
            const f32x4 q = qn;
            if (cq + 1 < ncq) qn = qp[(cq + 1) * 64];
#pragma unroll
            for (int b = 0; b < FOLD_NR / 8; ++b) {
                const f32x16 nxt0 = tile[(cq * (FOLD_NR / 8) + b + 1) * 2];
                const f32x16 nxt1 = tile[(cq * (FOLD_NR / 8) + b + 1) * 2 + 1];
                __builtin_amdgcn_sched_barrier(0);
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
        // a row with itself: +inf (only a tile that overlaps this wave's own rows can hold it)
        if (a.self_offset >= 0 && j0 < a.self_offset + q0 + 64 && j0 + FOLD_NR > a.self_offset + q0) {
#pragma unroll
            for (int t = 0; t < FOLD_NR / 16; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (j0 + 16 * t + r == selfj) acc[t][r] = __builtin_inff();
        }
        // minimum of each chunk of 32 columns (for select_rows_sparse); references past the end
        // of the set are zero rows in the packed copy and must not count
        if (a.M != nullptr) {
            const bool ragged = j0 + FOLD_NR > a.nr;
            float m0 = __builtin_inff(), m1 = __builtin_inff();
#pragma unroll
            for (int t = 0; t < FOLD_NR / 16; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float v = (ragged && j0 + 16 * t + r >= a.nr) ? __builtin_inff() : acc[t][r];
                    if (t < FOLD_NR / 32) m0 = fminf(m0, v);
                    else m1 = fminf(m1, v);
                }
            // Written 4 bytes at a time these would leave every 64-byte segment of the row half
            // filled for many tiles, and the L2 cannot hold that many open lines: it evicts them
            // partly written, which costs the memory a read-modify-write each (measured: 2.3 of
            // 16.3 ms).  So the wave collects 8 tiles (16 chunks, 64 bytes per row) in LDS first.
            float *slot = &s_min[w][lane * FB_PITCH + 2 * (int)(tj & 7)];
            slot[0] = m0;
            slot[1] = m1;
            if ((tj & 7) == 7 || tj + 1 == t1) {
                const int first_t = (int)max(tj & ~(int64_t)7, max(t0, TRI ? qg : (int64_t)0));
                float *mrow = a.M + myq * a.ldm + 2 * (tj & ~(int64_t)7);
                const float *src = &s_min[w][lane * FB_PITCH];
                if ((first_t & 7) == 0 && (tj & 7) == 7) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) *(f32x4 *)(mrow + 4 * i) = *(const f32x4 *)(src + 4 * i);
                } else {
                    for (int c = 2 * (first_t & 7); c <= 2 * (int)(tj & 7) + 1; ++c) mrow[c] = src[c];
                }
            }
        }
        // direct part: 16 columns at a time through the wave's LDS buffer
        {
            const int rr = lane >> 2, cc = (lane & 3) * 4;
            float *drow = a.D + (q0 + rr) * a.ldd + j0 + cc;
#pragma unroll
            for (int t = 0; t < FOLD_NR / 16; ++t) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 v = {acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]};
                    *(f32x4 *)(tr + lane * FD_PITCH + 4 * g) = v;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    f32x4 v = *(const f32x4 *)(tr + (rr + 16 * i) * FD_PITCH + cc);
                    *(f32x4 *)(drow + (int64_t)(16 * i) * a.ldd + 16 * t) = v;
                }
            }
        }
        if (MODE == DIST_RECT_MIRROR || (TRI && tj > qg)) {
            // a row address every lane agrees on plus a 32-bit lane offset (keeps the 64 store
            // addresses from taking two registers each)
            // (the address walks from row to row: 64 independent row addresses would be computed
            // ahead and spill the scalar registers that hold the reference operands)
            global_float *mrow = scalar_ptr(a.Dm + j0 * a.ldd);
            const uint32_t voff = (uint32_t)myq;
#pragma unroll
            for (int t = 0; t < FOLD_NR / 16; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    mrow[voff] = acc[t][r];
                    mrow += a.ldd;
                }
            // minima of the mirrored values: a chunk of row j's columns is one half of this wave's
            // queries.  16 rows at a time through the LDS buffer (row = reference, column = query);
            // lane 2 r + c reads chunk c of row r back and keeps the minimum.  Queries past the end
            // of the set go in as +inf.
            if (a.Mm != nullptr) {
                typedef float f32x2 __attribute__((ext_vector_type(2)));
                const bool qin = myq < a.nq;
#pragma unroll
                for (int t = 0; t < FOLD_NR / 16; ++t) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) tr[r * FM_PITCH + lane] = qin ? acc[t][r] : __builtin_inff();
                    if (lane < 32) {
                        const float *src = tr + (lane >> 1) * FM_PITCH + 32 * (lane & 1);
                        float m = __builtin_inff();
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            f32x2 v = *(const f32x2 *)(src + 2 * i);
                            m = fminf(m, fminf(v[0], v[1]));
                        }
                        a.Mm[(j0 + 16 * t + (lane >> 1)) * a.ldm + (q0 >> 5) + (lane & 1)] = m;
                    }
                }
            }
        }
    }
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

}  // namespace knn

#endif
