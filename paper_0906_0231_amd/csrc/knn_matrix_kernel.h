// The two-phase organisation of the paper (Sect. 5: Phase 1 writes the distance matrix,
// Sect. 6: Phase 2 selects per row) for problems where it is the cheaper one on this device:
// few rows and long lists, where the fused kernels spend more time merging candidates than
// multiplying, while an n x n matrix of a few GB costs HBM a millisecond or two to write and
// read back.  Phase 2 is select_rows.  Included by knn_kernels.hip only.
#ifndef KNN_MATRIX_KERNEL_H_
#define KNN_MATRIX_KERNEL_H_

namespace knn {

// ---------------------------------------------------------------------------
// knn_dist_qreg<DPAD, MODE>: Phase 1.  The matrix loop of knn_tiles_qreg (query operands in
// registers, 64 reference rows x 32 coordinates per step through LDS); the epilogue stores
// the tile instead of selecting from it:
//   D[q][j] = p(q, j) = c_j + sum Q'[q] R'[j]        (the value the fused kernels select on;
//                                                     finalize_rows adds the query's own term)
// DIST_TRIANGLE (knn_build with a symmetric distance, Sect. 3): a workgroup starts its sweep at
// its own diagonal block and every tile beyond it is stored twice, D[q][j] and, as row j sees
// the same pair, D[j][q] = (p - c_j) + c_q -- half the matrix products, the zig-zag of Sect. 4
// being unnecessary here because the sweeps are cut into chunks of equal length.  Stores to
// distinct elements need no ownership, so one launch covers the triangle.
// DIST_RECT_MIRROR: queries and references are two different row panels of one data set (a
// matrix too large to write out whole is walked panel pair by panel pair); every tile is stored
// twice, the mirrored values into the buffer of the transposed block.
// The entry of a row with itself is stored as +inf; columns past the end hold +inf (direct)
// or are never read (mirror).
// ---------------------------------------------------------------------------
// a pointer every lane agrees on, told to the compiler as such
typedef __attribute__((address_space(1))) float global_float;
__device__ __forceinline__ global_float *scalar_ptr(float *p)
{
    const u64 v = (u64)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (global_float *)(((u64)hi << 32) | lo);
}

constexpr int DT_PITCH = QG_TR + 4;               // floats per row of a wave's transposition buffer
constexpr int DB_PITCH = 20;                      // 16 chunk minima per row (+ pad, 16-byte aligned)
constexpr int DM_PITCH = 34;                      // the same buffer as 64 rows of 32 (+2) for the mirrored minima
static_assert(64 * DM_PITCH <= 32 * DT_PITCH, "the mirrored tile must fit the transposition buffer");
struct __attribute__((aligned(16))) DistSmem {
    float r[2][QG_RBUF];
    float c[2][QG_TR];                            // by tile parity: read again in the epilogue
    float tr[4][32 * DT_PITCH];                   // per wave: its 32 x 64 tile, query-major
    float mn[4][32 * DB_PITCH];                   // per wave: the chunk minima of 8 tiles for its 32 rows
    float u[2][QG_TR];                            // by tile parity: threshold + c of the tile's rows (test before the mirrored part)
};

template <int DPAD, int MODE>
__global__ __launch_bounds__(256, 2) void knn_dist_qreg(DistArgs a)
{
    constexpr int NK = DPAD / QG_DC;
    constexpr int NS = DPAD / 8;
    __shared__ DistSmem sm;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int h = lane >> 5;
    const int ql = lane & 31;

    // chunk-major numbering: consecutive workgroups (which go to the 8 XCDs in turn) are
    // consecutive query tiles of one chunk index.  In symmetric mode the chunks of high index
    // exist for the first query tiles only; numbered tile-major with a chunk count that is a
    // multiple of 8, every XCD would get its own chunk indices and the one with chunk 0 more
    // than twice the work of the last (measured: n = 65536 took 1.6 times too long).
    const int chunk = blockIdx.x / a.n_qtiles;
    const int qt = blockIdx.x - chunk * a.n_qtiles;
    // the diagonal block of query tile qt is reference tiles 2 qt and 2 qt + 1
    constexpr bool SYM = MODE != DIST_FULL;       // values are stored twice
    const int first = MODE == DIST_TRIANGLE ? 2 * qt : 0;
    const int mirror_from = MODE == DIST_TRIANGLE ? first + 2 : 0;   // first tile that is mirrored
    // chunk boundaries are the same for every query tile, so the workgroups of one chunk index
    // walk the same reference tiles at the same time and share them in the L2; the chunk that
    // holds the diagonal starts there, those below it leave at once
    const int rt0 = max(chunk * a.chunk, first);
    const int rt1 = min(chunk * a.chunk + a.chunk, a.n_rt);
    if (rt0 >= rt1) return;                       // whole workgroup

    const int64_t qbase = (int64_t)qt * TQ;
    const int64_t myq = qbase + 32 * w + ql;      // < nq_pad: D has that many rows
    const int64_t selfj = a.self_offset >= 0 ? a.self_offset + myq : -1;
    const bool qin = myq < a.nq;
    // the query's own term for the mirrored values; +inf past the end of the set, so that such a
    // column comes out as +inf and never lowers a chunk minimum
    const float cq = SYM ? (qin ? a.cQ[myq] : __builtin_inff()) : 0.f;
    // Rows that already have a full list (a matrix walked block by block): what cannot enter
    // the list is not stored.  tq: threshold of this lane's query row; tr_next / tr_cur: of
    // reference row 64 rt + lane, fetched a tile ahead.
    const float tq = a.tauQ != nullptr ? a.tauQ[min(myq, a.nq - 1)] : __builtin_inff();
    const bool filt_m = SYM && a.tauR != nullptr && a.Mm != nullptr;
    float tr_next = __builtin_inff(), tr_cur = __builtin_inff();

    f32x4 qreg[NS];
    {
        const float *qrow = a.Qp + min(myq, a.nq - 1) * a.ldq + h * 4;
#pragma unroll
        for (int s = 0; s < NS; ++s) qreg[s] = *(const f32x4 *)(qrow + s * 8);
    }

    const int lrow = tid >> 3, lunit = tid & 7;
    const int st_off = lrow * QG_DC + ((lunit ^ qg_swz(lrow)) << 2);
    f32x4 g0, g1;
    float gc = 0.f;
    auto issue = [&](int rt, int kc) __attribute__((always_inline)) {
        int64_t r0 = min((int64_t)rt * QG_TR + lrow, a.nr - 1);
        int64_t r1 = min((int64_t)rt * QG_TR + lrow + 32, a.nr - 1);
        g0 = *(const f32x4 *)(a.Rp + r0 * a.ldr + kc * QG_DC + lunit * 4);
        g1 = *(const f32x4 *)(a.Rp + r1 * a.ldr + kc * QG_DC + lunit * 4);
        if (kc == 0 && tid < QG_TR) gc = a.cR[(int64_t)rt * QG_TR + tid];
        if (kc == 0 && filt_m) tr_next = a.tauR[min((int64_t)rt * QG_TR + lane, a.nr - 1)];
    };
    auto stash = [&](int buf, int kc, int tb) __attribute__((always_inline)) {
        *(f32x4 *)&sm.r[buf][st_off] = g0;
        *(f32x4 *)&sm.r[buf][st_off + 32 * QG_DC] = g1;
        if (kc == 0 && tid < QG_TR) {
            sm.c[tb][tid] = gc;
            // u_j = tr_j + c_j, raised by more than the roundings of the two forms compared in the
            // epilogue can amount to (thread j of the first wave holds both)
            if (filt_m) sm.u[tb][tid] = (tr_next + gc) + 1e-6f * (fabsf(gc) + fabsf(tr_next));
        }
    };
    const int rbase0 = ql * QG_DC, rbase1 = (32 + ql) * QG_DC;
    const int sw = qg_swz(ql);

    f32x16 acc0, acc1;
    issue(rt0, 0);
    stash(0, 0, rt0 & 1);
    __syncthreads();

    int buf = 0;
    auto step = [&](auto kc_tag, int rt) __attribute__((always_inline)) {
        constexpr int kc = decltype(kc_tag)::value;
        constexpr bool last = kc == NK - 1;
        if (kc == 0) tr_cur = tr_next;            // this tile's; the fetch below is the next tile's
        // The chunk's last step fetches its own tile's first rows again instead of nothing: with
        // fetch and deposit unconditional the compiler knows which loads are pending where, and
        // puts no wait for them between the stores of the epilogue.
        issue(last ? min(rt + 1, rt1 - 1) : rt, last ? 0 : kc + 1);
        __builtin_amdgcn_sched_barrier(0);
        if (kc == 0) {
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
        // Deposit the next step's rows before the epilogue issues its stores: the loads were
        // issued before them, but how many stores follow is not known at compile time, so a wait
        // placed after them would be a wait for every store of the tile to be acknowledged.
        stash(buf ^ 1, last ? 0 : kc + 1, (rt + 1) & 1);
        if (last) {
            // register 4 gg + e of block t is reference row j0 + 32 t + 8 gg + 4 h + e
            const int64_t j0 = (int64_t)rt * QG_TR;
            const float INF = __builtin_inff();
            // Direct part, through the wave's own LDS buffer: in the accumulators a lane holds 4
            // consecutive columns of ITS row, so storing from there would write 32 bytes per row
            // and instruction; read back row-wise, 16 lanes cover the 256 bytes of a row.
            float *tw = &sm.tr[w][ql * DT_PITCH + 4 * h];
            // does the tile hold the entry of one of this wave's queries with itself?  (Only a
            // tile of the diagonal block can, and those are not mirrored.)
            const bool own = a.self_offset >= 0 && j0 < a.self_offset + qbase + 32 * w + 32 &&
                             j0 + QG_TR > a.self_offset + qbase + 32 * w;
            if (own) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (j0 + 8 * (i >> 2) + 4 * h + (i & 3) == selfj) acc0[i] = INF;
                    if (j0 + 32 + 8 * (i >> 2) + 4 * h + (i & 3) == selfj) acc1[i] = INF;
                }
            }
            // the minimum of each of the two chunks of 32 columns of this lane's row (the two
            // halves hold 16 columns of each)
            float min0 = acc0[0], min1 = acc1[0];
#pragma unroll
            for (int i = 1; i < 16; ++i) {
                min0 = fminf(min0, acc0[i]);
                min1 = fminf(min1, acc1[i]);
            }
            min0 = fminf(min0, __shfl_xor(min0, 32, 64));
            min1 = fminf(min1, __shfl_xor(min1, 32, 64));
            if (a.M != nullptr) {
                // chunk 2 rt is block 0, chunk 2 rt + 1 block 1: the first half writes the one,
                // the second the other.
                // Collected in LDS for 8 tiles (16 chunks = 64 bytes of the row) before they go
                // out: written 4 bytes at a time the half-filled lines outnumber what the L2 can
                // keep open, and every one evicted early costs the memory a read-modify-write
                sm.mn[w][ql * DB_PITCH + 2 * (rt & 7) + h] = h == 0 ? min0 : min1;
                if ((rt & 7) == 7 || rt + 1 == rt1) {
                    const int first_t = max(rt & ~7, rt0);
                    const int rowl = lane >> 1, part = (lane & 1) * 8;      // 32 rows x two halves of 8 chunks
                    float *mrow = a.M + (qbase + 32 * w + rowl) * a.ldm + 2 * (rt & ~7);
                    const float *src = &sm.mn[w][rowl * DB_PITCH];
                    if ((first_t & 7) == 0 && (rt & 7) == 7) {
                        *(f32x4 *)(mrow + part) = *(const f32x4 *)(src + part);
                        *(f32x4 *)(mrow + part + 4) = *(const f32x4 *)(src + part + 4);
                    } else {
                        for (int c = max(2 * (first_t & 7), part); c <= min(2 * (rt & 7) + 1, part + 7); ++c) mrow[c] = src[c];
                    }
                }
            }
            // bit r: row r of the wave's 32 can use its chunk (always, without thresholds)
            const uint32_t keep0 = (uint32_t)__ballot(min0 <= tq), keep1 = (uint32_t)__ballot(min1 <= tq);
            if (keep0 | keep1) {
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) {
                    *(f32x4 *)(tw + 8 * gg) = f32x4{acc0[4 * gg], acc0[4 * gg + 1], acc0[4 * gg + 2], acc0[4 * gg + 3]};
                    *(f32x4 *)(tw + 32 + 8 * gg) = f32x4{acc1[4 * gg], acc1[4 * gg + 1], acc1[4 * gg + 2], acc1[4 * gg + 3]};
                }
                const int rr = lane >> 4, cc = (lane & 15) * 4;
                const uint32_t keep = (lane & 8) ? keep1 : keep0;         // 8 lanes cover a chunk of a row
                float *drow = a.D + (qbase + 32 * w + rr) * a.ldd + j0 + cc;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    f32x4 v = *(const f32x4 *)&sm.tr[w][(rr + 4 * i) * DT_PITCH + cc];
                    if ((keep >> (rr + 4 * i)) & 1u) *(f32x4 *)(drow + (int64_t)(4 * i) * a.ldd) = v;
                }
            }
            if (SYM && rt >= mirror_from) {
                // Beyond the diagonal block: the same pairs as rows j see them; for a fixed
                // register the 32 lanes of a half hold 32 consecutive queries, 128 bytes of row j.
                // Addressed as a row address every lane agrees on plus a 32-bit lane offset, which
                // keeps the 32 store addresses from occupying two registers each across the loop.
                global_float *tbase = scalar_ptr(a.Dm + j0 * a.ldd);
                const uint32_t voff = (uint32_t)(4 * h * a.ldd + myq);       // the host keeps it below 2^32
                // The minima of the mirrored values: a chunk of row j's columns is this wave's 32
                // queries, i.e. one value per lane of a half -- a reduction across lanes for each
                // of the 32 register pairs.  Cheaper through the wave's LDS buffer: the values go in
                // row-major (row = reference j of the tile, column = query), lane j reads its row
                // back and keeps the minimum in its own registers.  (Columns past the end of the
                // set have c_q = +inf.)
                const bool want_min = a.Mm != nullptr;
                float *tm = &sm.tr[w][(4 * h) * DM_PITCH + ql];
                // One straight-line loop per case: with the two conditions tested inside, the
                // compiler left two branches per value in the loop, and a wave that branches 64
                // times next to one that streams matrix instructions waits for its instruction
                // fetches (measured: 4 300 cycles for this loop, median; 16 000 at the 90th
                // percentile).
                auto mirrored = [&](auto store_tag, auto lds_tag) __attribute__((always_inline)) {
                    constexpr bool STORE = decltype(store_tag)::value, LDS = decltype(lds_tag)::value;
#pragma unroll
                    for (int gg = 0; gg < 4; ++gg) {
                        f32x4 c0 = *(const f32x4 *)&sm.c[rt & 1][gg * 8 + h * 4];
                        f32x4 c1 = *(const f32x4 *)&sm.c[rt & 1][32 + gg * 8 + h * 4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float m0 = (acc0[4 * gg + e] - c0[e]) + cq;
                            const float m1 = (acc1[4 * gg + e] - c1[e]) + cq;
                            if (STORE) {
                                (tbase + (int64_t)(8 * gg + e) * a.ldd)[voff] = m0;
                                (tbase + (int64_t)(32 + 8 * gg + e) * a.ldd)[voff] = m1;
                            }
                            if (LDS) {
                                tm[(8 * gg + e) * DM_PITCH] = m0;
                                tm[(32 + 8 * gg + e) * DM_PITCH] = m1;
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);     // eight values at a time: no room for more at d = 256
                    }
                };
                // With thresholds, most tiles late in the walk hold nothing any row can use, and the
                // loop below (128 vector instructions, 64 LDS writes, then the minima) is the largest
                // part of the epilogue.  A cheaper test comes first.  Row j keeps a mirrored value
                // only if (acc - c_j) + c_q <= tr_j; with u_j = tr_j + c_j, raised by more than the
                // roundings of both forms can amount to, that needs acc - u_j + c_q <= ~0.  The u_j
                // came into LDS with the tile's c_j, the lanes read the values of their registers'
                // rows as they read c, and two chains of three-operand minima give the smallest
                // acc - u over the lane's 32 values.  If no lane finds one at or below -c_q, no row can use its
                // chunk: it is marked as such (a minimum of +inf: a row that has a threshold has a
                // full list, and the selection then compares the minima with that threshold only)
                // and nothing else is done.  No threshold yet (+inf), or rows past the end, never
                // pass this test; queries past the end have nothing to keep.
                bool none = false;
                if (filt_m) {
                    float ma = INF, mb = INF;
#pragma unroll
                    for (int gg = 0; gg < 4; ++gg) {
                        f32x4 u0 = *(const f32x4 *)&sm.u[rt & 1][gg * 8 + h * 4];
                        f32x4 u1 = *(const f32x4 *)&sm.u[rt & 1][32 + gg * 8 + h * 4];
                        ma = fminf(ma, fminf(acc0[4 * gg + 0] - u0[0], acc0[4 * gg + 1] - u0[1]));
                        mb = fminf(mb, fminf(acc0[4 * gg + 2] - u0[2], acc0[4 * gg + 3] - u0[3]));
                        ma = fminf(ma, fminf(acc1[4 * gg + 0] - u1[0], acc1[4 * gg + 1] - u1[1]));
                        mb = fminf(mb, fminf(acc1[4 * gg + 2] - u1[2], acc1[4 * gg + 3] - u1[3]));
                    }
                    none = __ballot(qin && !(fminf(ma, mb) + cq > 1e-6f * fabsf(cq))) == 0;
                }
                if (none) {
                    a.Mm[(j0 + lane) * a.ldm + (qbase >> 5) + w] = INF;
                } else if (filt_m) {                          // (implies want_min)
                    mirrored(std::false_type{}, std::true_type{});
                } else if (want_min) {
                    mirrored(std::true_type{}, std::true_type{});
                } else {
                    mirrored(std::true_type{}, std::false_type{});
                }
                if (want_min && !none) {
                    typedef float f32x2 __attribute__((ext_vector_type(2)));
                    const float *tr_row = &sm.tr[w][lane * DM_PITCH];
                    float m = INF;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        f32x2 v = *(const f32x2 *)(tr_row + 2 * i);
                        m = fminf(m, fminf(v[0], v[1]));
                    }
                    a.Mm[(j0 + lane) * a.ldm + (qbase >> 5) + w] = m;
                    if (filt_m) {
                        // bit j: row j0 + j can use the wave's chunk; the stores wait for this
                        u64 keep = __ballot(m <= tr_cur);
                        // The rows kept (one or two of the 64, typically) are copied out of the LDS
                        // buffer, where each lies as 32 consecutive values: two rows per pass, one
                        // per half of the wave.  (64 stores each under its own test of a mask bit
                        // were 64 branches, which next to a wave that streams matrix instructions
                        // cost far more than they look.)
                        while (keep) {
                            const int r0 = __builtin_ctzll(keep);
                            keep &= keep - 1;
                            int r1 = -1;
                            if (keep) {
                                r1 = __builtin_ctzll(keep);
                                keep &= keep - 1;
                            }
                            const int r = h == 0 ? r0 : r1;
                            if (r >= 0)
                                a.Dm[(j0 + r) * a.ldd + qbase + 32 * w + ql] = sm.tr[w][r * DM_PITCH + ql];
                        }
                    }
                }
            }
        }
        __syncthreads();
        buf ^= 1;
    };
    for (int rt = rt0; rt < rt1; ++rt) for_each_step<NK>(step, rt);
}

// ---------------------------------------------------------------------------
// knn_dist_stream<MODE>: Phase 1 for any d -- the matrix loop of knn_tiles (both operands
// through LDS 16 coordinates at a time, tile 128 x 128, four accumulator blocks per wave), the
// epilogue a store as in knn_dist_qreg.  The diagonal block of query tile t is reference tile t.
// The direct part leaves through a per-wave LDS buffer one 32 x 32 block at a time (128-byte
// row segments); in the mirrored part the 32 lanes of a half hold 32 consecutive queries.
// ---------------------------------------------------------------------------
constexpr int DS_PITCH = 36;                      // floats per row of the transposition buffer

struct __attribute__((aligned(16))) DistStreamSmem {
    float q[2][TQ * LSTR];
    float r[2][TR * LSTR];
    float c[2][TR];                               // by tile parity: read again in the epilogue
    float tr[4][32 * DS_PITCH];
    float mn[4][32 * DB_PITCH];                   // per wave: the chunk minima of 4 tiles for its 32 rows
};
static_assert(32 * DM_PITCH <= 32 * DS_PITCH, "a mirrored block must fit the transposition buffer");

template <int MODE>
__global__ __launch_bounds__(256, 2) void knn_dist_stream(DistArgs a)
{
    __shared__ DistStreamSmem sm;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int h = lane >> 5;
    const int ql = lane & 31;
    constexpr bool SYM = MODE != DIST_FULL;

    const int chunk = blockIdx.x / a.n_qtiles;    // chunk-major, see knn_dist_qreg
    const int qt = blockIdx.x - chunk * a.n_qtiles;
    const int first = MODE == DIST_TRIANGLE ? qt : 0;
    const int mirror_from = MODE == DIST_TRIANGLE ? first + 1 : 0;
    const int rt0 = max(chunk * a.chunk, first);  // a.n_rt, a.chunk: in tiles of 128 reference rows here
    const int rt1 = min(chunk * a.chunk + a.chunk, a.n_rt);
    if (rt0 >= rt1) return;                       // whole workgroup
    const int nk = a.dpad / DC;

    const int64_t qbase = (int64_t)qt * TQ;
    const int64_t myq = qbase + 32 * w + ql;
    const int64_t selfj = a.self_offset >= 0 ? a.self_offset + myq : -1;
    const float cq = SYM ? a.cQ[min(myq, a.nq - 1)] : 0.f;
    const bool qin = myq < a.nq;
    // Rows that already have a full list (a matrix walked block by block): what cannot enter the
    // list is not stored, as in knn_dist_qreg.  tq: threshold of this lane's query row; trv[t]: of
    // reference row 128 rt + 32 t + (lane & 31), fetched one step before the tile's last.
    const float tq = a.tauQ != nullptr ? a.tauQ[min(myq, a.nq - 1)] : __builtin_inff();
    const bool filt_m = SYM && a.tauR != nullptr && a.Mm != nullptr;
    float trv[4] = {0.f, 0.f, 0.f, 0.f};

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
        if (kc == nk - 1 && filt_m) {
#pragma unroll
            for (int t = 0; t < 4; ++t) trv[t] = a.tauR[min((int64_t)rt * TR + 32 * t + ql, a.nr - 1)];
        }
    };
    auto stash = [&](int buf, int kc, int tb) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NPASS; ++i) {
            *(f32x4 *)&sm.q[buf][(lrow + i * ROWS_PER_PASS) * LSTR + lcol] = gq[i];
            *(f32x4 *)&sm.r[buf][(lrow + i * ROWS_PER_PASS) * LSTR + lcol] = gr[i];
        }
        if (kc == 0 && tid < TR) sm.c[tb][tid] = gc;
    };

    f32x16 acc[4];
    const int total = (rt1 - rt0) * nk;
    issue(rt0, 0);
    stash(0, 0, rt0 & 1);
    __syncthreads();

    int rt = rt0, kc = 0;
    for (int it = 0; it < total; ++it) {
        const int buf = it & 1;
        int nrt = rt, nkc = kc + 1;
        if (nkc == nk) { nkc = 0; nrt = rt + 1; }
        // The last step fetches its own operands again instead of nothing: with the fetch and the
        // deposit unconditional the compiler knows at the top of a step that no load is pending,
        // and the address arithmetic does not wait for the stores of the tile before.
        if (it + 1 == total) { nrt = rt; nkc = kc; }
        issue(nrt, nkc);

        if (kc == 0) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 cv = *(const f32x4 *)&sm.c[rt & 1][t * 32 + g * 8 + h * 4];
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

        // deposit the next step's operands before the stores of the epilogue are issued: the
        // wait for the loads then does not include them
        stash(buf ^ 1, nkc, nrt & 1);
        if (kc == nk - 1) {
            // register 4 g + e of block t is reference row j0 + 32 t + 8 g + 4 h + e
            const int64_t j0 = (int64_t)rt * TR;
            const float INF = __builtin_inff();
            const bool own = a.self_offset >= 0 && j0 < a.self_offset + qbase + 32 * w + 32 &&
                             j0 + TR > a.self_offset + qbase + 32 * w;
            float *tw = &sm.tr[w][ql * DS_PITCH + 4 * h];
            const int rr = lane >> 3, cc = (lane & 7) * 4;
            float *drow = a.D + (qbase + 32 * w + rr) * a.ldd + j0 + cc;
            if (own) {                            // (a tile with a wave's own rows is never mirrored)
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (j0 + 32 * t + 8 * (i >> 2) + 4 * h + (i & 3) == selfj) acc[t][i] = INF;
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                // chunk 4 rt + t is block t; its 32 columns sit in the row's two lanes
                float dmin = min16(acc[t]);
                dmin = fminf(dmin, __shfl_xor(dmin, 32, 64));
                // collected in LDS for 4 tiles (16 chunks, 64 bytes of the row), see knn_dist_qreg
                if (a.M != nullptr && h == 0) sm.mn[w][ql * DB_PITCH + 4 * (rt & 3) + t] = dmin;
                // bit r: row r of the wave's 32 can use this chunk (always, without thresholds)
                const uint32_t keep = (uint32_t)__ballot(dmin <= tq);
                if (keep) {
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        *(f32x4 *)(tw + 8 * g) = f32x4{acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        f32x4 v = *(const f32x4 *)&sm.tr[w][(rr + 8 * i) * DS_PITCH + cc];
                        if ((keep >> (rr + 8 * i)) & 1u) *(f32x4 *)(drow + (int64_t)(8 * i) * a.ldd + 32 * t) = v;
                    }
                }
            }
            if (a.M != nullptr && ((rt & 3) == 3 || rt + 1 == rt1)) {
                const int first_t = max(rt & ~3, rt0);
                const int rowl = lane >> 1, part = (lane & 1) * 8;
                float *mrow = a.M + (qbase + 32 * w + rowl) * a.ldm + 4 * (rt & ~3);
                const float *src = &sm.mn[w][rowl * DB_PITCH];
                if ((first_t & 3) == 0 && (rt & 3) == 3) {
                    *(f32x4 *)(mrow + part) = *(const f32x4 *)(src + part);
                    *(f32x4 *)(mrow + part + 4) = *(const f32x4 *)(src + part + 4);
                } else {
                    for (int c = max(4 * (first_t & 3), part); c <= min(4 * (rt & 3) + 3, part + 7); ++c) mrow[c] = src[c];
                }
            }
            if (SYM && rt >= mirror_from) {
                global_float *tbase = scalar_ptr(a.Dm + j0 * a.ldd);
                const uint32_t voff = (uint32_t)(4 * h * a.ldd + myq);       // the host keeps it below 2^32
                // minima of the mirrored values: one block of 32 reference rows at a time through
                // the wave's LDS buffer (row = reference, column = query), lane r reads row r back
                const bool want_min = a.Mm != nullptr;
                float *tm = &sm.tr[w][(4 * h) * DM_PITCH + ql];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if (filt_m) {
                        // thresholds: the values go to LDS only, the minimum of each row decides
                        // whether the row's 32 values are stored at all
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            f32x4 cv = *(const f32x4 *)&sm.c[rt & 1][t * 32 + g * 8 + h * 4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float m = (acc[t][4 * g + e] - cv[e]) + cq;
                                tm[(8 * g + e) * DM_PITCH] = qin ? m : INF;
                            }
                        }
                        typedef float f32x2 __attribute__((ext_vector_type(2)));
                        const float *tr_row = &sm.tr[w][(lane & 31) * DM_PITCH];
                        float m = INF;
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            f32x2 v = *(const f32x2 *)(tr_row + 2 * i);
                            m = fminf(m, fminf(v[0], v[1]));
                        }
                        if (lane < 32) a.Mm[(j0 + 32 * t + lane) * a.ldm + (qbase >> 5) + w] = m;
                        // bit r: row j0 + 32 t + r can use the wave's chunk
                        uint32_t keep = (uint32_t)__ballot(m <= trv[t]);
                        // the rows kept are copied out of the LDS buffer, two per pass (see knn_dist_qreg)
                        while (keep) {
                            const int r0 = __builtin_ctz(keep);
                            keep &= keep - 1;
                            int r1 = -1;
                            if (keep) {
                                r1 = __builtin_ctz(keep);
                                keep &= keep - 1;
                            }
                            const int r = h == 0 ? r0 : r1;
                            if (r >= 0)
                                a.Dm[(j0 + 32 * t + r) * a.ldd + qbase + 32 * w + ql] = sm.tr[w][r * DM_PITCH + ql];
                        }
                        continue;
                    }
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        f32x4 cv = *(const f32x4 *)&sm.c[rt & 1][t * 32 + g * 8 + h * 4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float m = (acc[t][4 * g + e] - cv[e]) + cq;
                            (tbase + (int64_t)(32 * t + 8 * g + e) * a.ldd)[voff] = m;
                            if (want_min) tm[(8 * g + e) * DM_PITCH] = qin ? m : INF;
                        }
                    }
                    if (want_min && lane < 32) {
                        typedef float f32x2 __attribute__((ext_vector_type(2)));
                        const float *tr_row = &sm.tr[w][lane * DM_PITCH];
                        float m = INF;
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            f32x2 v = *(const f32x2 *)(tr_row + 2 * i);
                            m = fminf(m, fminf(v[0], v[1]));
                        }
                        a.Mm[(j0 + 32 * t + lane) * a.ldm + (qbase >> 5) + w] = m;
                    }
                }
            }
        }

        __syncthreads();
        rt = nrt;
        kc = nkc;
    }
}

}  // namespace knn

#endif
