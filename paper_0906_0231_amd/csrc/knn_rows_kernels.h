// Per-row kernels bound by HBM: prep_rows (norms and scaled copies), select_rows (batched partial
// sort of a materialised matrix, paper Sect. 6), finalize_rows (merge of partial lists, re-score,
// final order), reduce_max.  Included by knn_kernels.hip only.
#ifndef KNN_ROWS_KERNELS_H_
#define KNN_ROWS_KERNELS_H_

namespace knn {

// ---------------------------------------------------------------------------
// Column means (knn_options_t.center): the vector subtracted from every row before the expanded
// form is taken, so that data far from the origin does not lose its distances in the rounding of
// |q|^2 + |r|^2 - 2 q.r.  col_sum: a thread per column, the rows dealt over blockIdx.y, partial
// sums in double added atomically; col_mean: the division, zero beyond d.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void col_zero(double *sums, int32_t dpad)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c < dpad) sums[c] = 0.0;
}

__global__ __launch_bounds__(256) void col_sum(const float *X, int64_t n, int32_t d, double *sums)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= d) return;
    double s = 0.0;
    for (int64_t r = blockIdx.y; r < n; r += gridDim.y) s += (double)X[r * d + c];
    atomicAdd(&sums[c], s);
}

__global__ __launch_bounds__(256) void col_mean(const double *sums, int64_t n, int32_t d, int32_t dpad, float *mu)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c < dpad) mu[c] = c < d ? (float)(sums[c] / (double)n) : 0.f;
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
                if (a.b_out) a.b_out[row] = 0xffffffffu;
            }
            continue;
        }
        // centred value of coordinate c: the difference is exact in double and rounded once
        auto val = [&](int c) __attribute__((always_inline)) {
            if (root) return sqrtf(x[c]);
            return a.mu != nullptr ? (float)((double)x[c] - (double)a.mu[c]) : x[c];
        };
        float s = 0.f;
        for (int c = lane; c < a.d; c += 64) {
            float v = val(c);
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
            for (int c = lane; c < a.dpad; c += 64) o[c] = c < a.d ? qscale * val(c) : 0.f;
        }
        if (a.r_out) {
            float *o = a.r_out + row * (int64_t)a.dpad;
            for (int c = lane; c < a.dpad; c += 64) o[c] = c < a.d ? rscale * val(c) : 0.f;
        }
        if (lane == 0) {
            if (a.c_out) a.c_out[row] = cval;
            if (a.s_out) a.s_out[row] = s;
            if (a.b_out) a.b_out[row] = 0xffffffffu;
        }
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
    // resume: the row's list holds the result of earlier calls over other column blocks
    u64 *out = a.lists + ((int64_t)seg * a.m + row) * a.kcap;
    for (int i = lane; i < a.kcap; i += 64) L[i] = a.resume ? out[i] : KEY_INF;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");

    const float INF = __builtin_inff();
    u64 tau_key = a.resume ? L[a.k - 1] : KEY_INF;
    float tau_p = tau_key == KEY_INF ? INF : ord2f((uint32_t)(tau_key >> 32));
    int count = 0;                                // queued candidates (wave-uniform)

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
                    const u64 key = make_key(p, (int32_t)(col + a.col0));
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
    for (int i = lane; i < a.kcap; i += 64) out[i] = L[i];
    if (a.tau_out != nullptr && lane == 0)
        a.tau_out[row] = tau_key == KEY_INF ? __builtin_inff() : ord2f((uint32_t)(tau_key >> 32));
}

// ---------------------------------------------------------------------------
// read_only: calibration.  Reads a buffer once, the way select_rows reads its rows (every wave
// a contiguous range, 8 KB per step, every lane eight 16-byte loads in flight, consecutive
// lanes consecutive addresses), keeps the minimum and does nothing else: the read rate this
// device's memory sustains, to put beside the nominal peak.  One value per workgroup goes to
// the sink.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void read_only(const float *buf, int64_t n_pieces, int64_t pieces_per_wave,
                                                 float *sink)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t p0 = wave * pieces_per_wave, p1 = min(p0 + pieces_per_wave, n_pieces);
    float m = __builtin_inff();
    for (int64_t piece = p0; piece < p1; ++piece) {                    // pieces of SEL_CHUNK floats
        const f32x4 *src = (const f32x4 *)(buf + piece * SEL_CHUNK) + lane;
        f32x4 v[SEL_LOADS];
#pragma unroll
        for (int j = 0; j < SEL_LOADS; ++j) v[j] = src[j * 64];
#pragma unroll
        for (int j = 0; j < SEL_LOADS; ++j) m = fminf(m, fminf(fminf(v[j][0], v[j][1]), fminf(v[j][2], v[j][3])));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fminf(m, __shfl_xor(m, o, 64));
    if (threadIdx.x == 0) sink[blockIdx.x & 1023] = m;
}

// ---------------------------------------------------------------------------
// select_rows_sparse: select_rows for a matrix that comes with the minimum of every chunk of 32
// columns (written by the distance kernel on the way).  One wave per (row, column segment):
//   1. the k-th smallest of (a sample of) the row's chunk minima bounds the k-th smallest value
//      from above (k chunks hold at least one value each that is no larger), so
//   2. only chunks whose minimum is within the bound (and within the list's own threshold as
//      it tightens) are read, eight chunks per wave load; for k << n / 32 that is a small part
//      of the row, and the kernel reads n / 8 + a few k * 128 bytes per row instead of 4 n.
// Same list, queue and merge as select_rows; ties, `resume` and `col0` likewise.  A chunk whose
// minimum is above the threshold the row's list had before this call is never read -- the
// distance kernel relies on that and may have left such a chunk unwritten (DistArgs.tauQ).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void select_rows_sparse(SelectArgs a)
{
    __shared__ u64 sList[4][KNN_MAX_KCAP];
    __shared__ u64 sQueue[4][64];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int64_t gw = (int64_t)blockIdx.x * 4 + w;
    if (gw >= a.m * a.S) return;                  // whole wave; no barriers in this kernel
    const int64_t row = gw / a.S;
    const int seg = (int)(gw - row * a.S);
    const int64_t c0 = (int64_t)seg * a.seg;      // multiple of 1024
    const int64_t c1 = min(c0 + a.seg, a.n);
    const float *Arow = a.A + row * a.lda;
    const float *Mrow = a.M + row * a.ldm;
    const int64_t ch0 = c0 >> 5, ch1 = (c1 + 31) >> 5;
    u64 *L = &sList[w][0];
    u64 *Q = &sQueue[w][0];
    const float INF = __builtin_inff();
    int count = 0;                                // queued candidates (wave-uniform)

    // ---- step 1: a bound from the chunk minima.  Any k chunks whose minima are <= b prove that
    // the k-th smallest value is <= b.  Every lane keeps the 4 smallest minima of the chunks it
    // reads (256 candidates in registers, all from different chunks); the bound is the k-th
    // smallest of those -- a little looser than the k-th smallest of all minima (a lane that
    // holds more than 4 of the true k smallest drops some), at a small part of the cost of
    // selecting exactly (which took more than half of this kernel's time).
    // (A list that is continued and already full brings its own threshold: the minima are then
    // read once, in step 2 only.)
    u64 *out = a.lists + ((int64_t)seg * a.m + row) * a.kcap;
    const bool full = a.resume && out[a.k - 1] != KEY_INF;
    float bound = INF;
    if (ch1 - ch0 >= a.k && !full) {
        float s0 = INF, s1 = INF, s2 = INF, s3 = INF;            // ascending
        // 1024 minima per step (four 16-byte loads per lane in flight: one wave per row has little
        // else to hide the latency behind)
        for (int64_t g0 = ch0; g0 < ch1; g0 += 1024) {
            f32x4 m[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t g = g0 + j * 256 + lane * 4;
                m[j] = g < ch1 ? *(const f32x4 *)(Mrow + g) : f32x4{INF, INF, INF, INF};
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t g = g0 + j * 256 + lane * 4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float v = g + e < ch1 ? m[j][e] : INF;
                    float t;
                    t = fminf(s0, v); v = fmaxf(s0, v); s0 = t;
                    t = fminf(s1, v); v = fmaxf(s1, v); s1 = t;
                    t = fminf(s2, v); v = fmaxf(s2, v); s2 = t;
                    s3 = fminf(s3, v);
                }
            }
        }
        // rank: for each kept value, how many of the 256 are <= it
        int c0 = 0, c1 = 0, c2 = 0, c3 = 0;
#pragma unroll 1
        for (int l = 0; l < 64; ++l) {
            const float x0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s0), l));
            const float x1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s1), l));
            const float x2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s2), l));
            const float x3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s3), l));
            c0 += (x0 <= s0) + (x1 <= s0) + (x2 <= s0) + (x3 <= s0);
            c1 += (x0 <= s1) + (x1 <= s1) + (x2 <= s1) + (x3 <= s1);
            c2 += (x0 <= s2) + (x1 <= s2) + (x2 <= s2) + (x3 <= s2);
            c3 += (x0 <= s3) + (x1 <= s3) + (x2 <= s3) + (x3 <= s3);
        }
        float b = INF;
        if (c0 >= a.k) b = fminf(b, s0);
        if (c1 >= a.k) b = fminf(b, s1);
        if (c2 >= a.k) b = fminf(b, s2);
        if (c3 >= a.k) b = fminf(b, s3);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) b = fminf(b, __shfl_xor(b, o, 64));
        bound = b;
    }

    // ---- step 2: the chunks within the bound
    for (int i = lane; i < a.kcap; i += 64) L[i] = a.resume ? out[i] : KEY_INF;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    u64 tau_key = a.resume ? L[a.k - 1] : KEY_INF;
    float tau_p = tau_key == KEY_INF ? bound : fminf(bound, ord2f((uint32_t)(tau_key >> 32)));

    auto flush = [&]() __attribute__((always_inline)) {
        if (count == 0) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        u64 nt = merge_one(L, a.kcap, a.k, Q, count, lane);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        tau_key = nt;
        tau_p = nt == KEY_INF ? bound : fminf(bound, ord2f((uint32_t)(nt >> 32)));
        count = 0;
    };

    const int sub = lane >> 3;                    // which of the 8 chunks of a wave load
    const int part = (lane & 7) * 4;              // which 4 of its 32 columns
    for (int64_t g0 = ch0; g0 < ch1; g0 += 1024) {
      // the minima of 1024 chunks: lane l holds chunks g0 + 256 j + 4 l + e as mm[4 j + e]
      float mm[16];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
          const int64_t g = g0 + j * 256 + lane * 4;
          const f32x4 m = g < ch1 ? *(const f32x4 *)(Mrow + g) : f32x4{INF, INF, INF, INF};
#pragma unroll
          for (int e = 0; e < 4; ++e) mm[4 * j + e] = g + e < ch1 ? m[e] : INF;
      }
#pragma unroll 1
      for (int t = 0; t < 16; ++t) {
        const float mc = mm[0];
#pragma unroll
        for (int i = 0; i < 15; ++i) mm[i] = mm[i + 1];
        const int64_t base = g0 + (t >> 2) * 256 + (t & 3);      // lane l: chunk base + 4 l
        u64 todo = __ballot(mc <= tau_p);
        while (todo) {
            // the next (up to) 8 marked chunks, one per group of 8 lanes
            int pick = -1;
            u64 rest = todo;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int b = rest ? __builtin_ctzll(rest) : -1;
                if (rest) rest &= rest - 1;
                if (sub == i) pick = b;
            }
            todo = rest;
            // the threshold may have tightened since the chunk was marked
            const float pm = __shfl(mc, pick < 0 ? 0 : pick, 64);
            const bool live = pick >= 0 && pm <= tau_p;
            const int64_t col = ((base + 4 * (pick < 0 ? 0 : pick)) << 5) + part;
            f32x4 v = {INF, INF, INF, INF};
            if (live) {
                if (a.vec4 && col + 3 < c1) {
                    v = *(const f32x4 *)(Arow + col);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = col + e < c1 ? Arow[col + e] : INF;
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float p = v[e];
                const bool c = live && p <= tau_p;
                if (__ballot(c)) {
                    const u64 key = make_key(p, (int32_t)(col + e + a.col0));
                    const bool pass = c && key < tau_key && col + e < c1;
                    u64 bal = __ballot(pass);
                    int np = __popcll(bal);
                    if (np) {
                        if (count + np > 64) flush();     // entries already chosen stay valid candidates
                        int pos = count + __popcll(bal & ((1ull << lane) - 1ull));
                        if (pass) Q[pos] = key;
                        count += np;
                    }
                }
            }
            // (while the list is short of k the bound does the filtering; no need to merge eagerly)
            if (count >= 32 || (tau_key == KEY_INF && bound == INF)) flush();
        }
      }
    }
    flush();
    for (int i = lane; i < a.kcap; i += 64) out[i] = L[i];
    if (a.tau_out != nullptr && lane == 0)
        a.tau_out[row] = tau_key == KEY_INF ? __builtin_inff() : ord2f((uint32_t)(tau_key >> 32));
}

// ---------------------------------------------------------------------------
// finalize_rows: one wave per query.
// ---------------------------------------------------------------------------


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

// sum over the 16 lanes of a lane's quarter of the wave
__device__ __forceinline__ double group16_sum_f64(double v)
{
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// sqrt of a non-negative float as a double, to about 1e-13 relative: the hardware's single
// precision reciprocal square root (1 ulp) and one Newton step in double.  With r = (1 + e)/sqrt(v),
// h = v r and 1 - h r = -2e - e^2, h (1 + (1 - h r)/2) = sqrt(v) (1 - 1.5 e^2).  The library
// routine for double costs three times as much, and the Hellinger re-pricing takes one root per
// coordinate and winner.  Zero is exact; denormals (and NaN) take the library routine.
__device__ __forceinline__ double sqrt_of_float(float v)
{
    if (v == 0.f) return 0.0;
    if (!(v >= 1.17549435e-38f)) return sqrt((double)v);
    const double r = (double)__builtin_amdgcn_rsqf(v);
    const double h = (double)v * r;
    return fma(0.5 * h, fma(-h, r, 1.0), h);
}

__global__ __launch_bounds__(64) void finalize_rows(FinArgs a)
{
    // sized by the launcher to what this call needs (S * kcap keys rounded up to a power of two,
    // then k rounded up likewise): with one list per query that is 2 KB instead of 17, and three
    // times as many queries in flight per CU for the row gathers below
    extern __shared__ u64 fin_lds[];
    const int lane = threadIdx.x;
    // lq: position of the query's lists; q: the query's row (they differ in the second pass over a
    // compacted subset of the rows)
    const int64_t lq = blockIdx.x;
    if (a.nq_dev != nullptr && lq >= *a.nq_dev) return;
    const int64_t q = a.row_map != nullptr ? a.row_map[lq] : lq;

    const int nin = a.S * a.kcap;
    int npow = 1;
    while (npow < nin) npow <<= 1;
    u64 *keys = fin_lds;
    u64 *outk = fin_lds + npow;
    for (int i = lane; i < npow; i += 64) {
        u64 v = KEY_INF;
        if (i < nin) {
            int s = i / a.kcap, e = i - s * a.kcap;
            v = a.lists[((int64_t)s * a.nq_pad + lq) * a.kcap + e];
        }
        keys[i] = v;
    }
    __syncthreads();
    if (a.S > 1) bitonic_sort_lds(keys, npow, lane);

    // entries that are priced again below: the k winners, or (filter-and-refine) the first krs > k
    const int kr = a.krs > 0 ? a.krs : a.k;
    int kpow = 1;
    while (kpow < kr) kpow <<= 1;
    for (int i = lane; i < kpow; i += 64) outk[i] = KEY_INF;
    __syncthreads();

    // Re-pricing: the k winners are priced again from the original rows, accumulating in double
    // (a direct sum of squared differences, 1 - cos from the three sums, ...), so the reported
    // value carries neither the cancellation of |u|^2+|v|^2-2u.v nor that of 1-cos in fp32.
    // n*k*d work, bound by the latency of the row gathers: the wave is cut into four groups of 16
    // lanes that price four winners at a time.
    const int g16 = lane >> 4, gl = lane & 15;
    if (a.mode == FIN_RESCORE_L1 || a.mode == FIN_RESCORE_LINF || a.mode == FIN_RESCORE_KL) {
        const float *x = a.Q + q * (int64_t)a.d;
        for (int r0 = 0; r0 < a.k; r0 += 4) {
            const int r = r0 + g16;
            const int32_t j = r < a.k ? (int32_t)(uint32_t)keys[r] : -1;
            const bool ok = j >= 0 && j < a.nr;    // else an unfilled slot (cannot happen for k <= nr - self)
            const float *y = a.R + (int64_t)(ok ? j : 0) * a.d;
            double s = 0.0;
            if (ok) {
                for (int c = gl; c < a.d; c += 16) {
                    double ud = (double)x[c], vd = (double)y[c];
                    if (a.mode == FIN_RESCORE_L1) s += fabs(ud - vd);
                    else if (a.mode == FIN_RESCORE_LINF) s = fmax(s, fabs(ud - vd));
                    else if (ud > 0.0) s += ud * log(ud / vd);
                }
            }
            if (a.mode == FIN_RESCORE_LINF) {
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) s = fmax(s, __shfl_xor(s, o, 64));
            } else {
                s = group16_sum_f64(s);
            }
            if (gl == 0 && r < a.k) outk[r] = ok ? make_key((float)s, j) : KEY_INF;
        }
    } else if (a.mode == FIN_RESCORE_SQ || a.mode == FIN_RESCORE_COS || a.mode == FIN_RESCORE_HEL) {
        const float *x = a.Q + q * (int64_t)a.d;
        const bool cosine = a.mode == FIN_RESCORE_COS;
        const bool root = a.mode == FIN_RESCORE_HEL;
        // Hellinger: the square roots of the query's own coordinates are the same for every
        // winner; a lane takes them once (its 4 of every 64 coordinates, up to d = 256)
        const bool pre = root && a.vec4 && a.d <= 256;
        double xs[4][4];
        if (pre) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = gl * 4 + 64 * i;
                f32x4 u = {0.f, 0.f, 0.f, 0.f};
                if (c < a.d) u = *(const f32x4 *)(x + c);
#pragma unroll
                for (int e = 0; e < 4; ++e) xs[i][e] = sqrt_of_float(u[e]);
            }
        }
        for (int r0 = 0; r0 < kr; r0 += 4) {
            const int r = r0 + g16;
            const int32_t j = r < kr ? (int32_t)(uint32_t)keys[r] : -1;
            const bool ok = j >= 0 && j < a.nr;
            const float *y = a.R + (int64_t)(ok ? j : 0) * a.d;
            double s = 0.0, uu = 0.0, vv = 0.0;
            if (ok && pre) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int c = gl * 4 + 64 * i;
                    if (c < a.d) {
                        f32x4 v = *(const f32x4 *)(y + c);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            double t = xs[i][e] - sqrt_of_float(v[e]);
                            s = fma(t, t, s);
                        }
                    }
                }
            } else if (ok && a.vec4) {
                for (int c = gl * 4; c < a.d; c += 64) {
                    f32x4 u = *(const f32x4 *)(x + c), v = *(const f32x4 *)(y + c);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        double ud = (double)u[e], vd = (double)v[e];
                        if (cosine) {
                            s = fma(ud, vd, s);
                            uu = fma(ud, ud, uu);
                            vv = fma(vd, vd, vv);
                        } else {
                            double t = root ? sqrt_of_float(u[e]) - sqrt_of_float(v[e]) : ud - vd;
                            s = fma(t, t, s);
                        }
                    }
                }
            } else if (ok) {
                for (int c = gl; c < a.d; c += 16) {
                    double ud = (double)x[c], vd = (double)y[c];
                    if (cosine) {
                        s = fma(ud, vd, s);
                        uu = fma(ud, ud, uu);
                        vv = fma(vd, vd, vv);
                    } else {
                        double t = root ? sqrt_of_float(x[c]) - sqrt_of_float(y[c]) : ud - vd;
                        s = fma(t, t, s);
                    }
                }
            }
            s = group16_sum_f64(s);
            if (cosine) {
                uu = group16_sum_f64(uu);
                vv = group16_sum_f64(vv);
                s = (uu == 0.0 || vv == 0.0) ? 1.0 : 1.0 - s / (sqrt(uu) * sqrt(vv));
                if (s < 0.0) s = 0.0;
            }
            if (gl == 0 && r < kr) outk[r] = ok ? make_key((float)s, j) : KEY_INF;
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
        const int32_t j = (int32_t)(uint32_t)key;
        a.idx[q * a.k + r] = j;
        // knn_select returns copies of the matrix entries: taken from the matrix itself, since a
        // key does not keep the sign of a zero (keys of -0 and +0 tie, as the values do)
        a.dist[q * a.k + r] = (a.mode == FIN_SELECT && a.Q != nullptr) ? a.Q[q * a.nr + j] : ord2f((uint32_t)(key >> 32));
    }
    if (a.krs > 0 && a.uncert != nullptr) {
        // Certificate of the filter.  The lists hold, by approximate value p~, the krs smallest of
        // ALL references, so a reference j outside them has p~_j >= t~ (the krs-th kept value)
        // and a true value p_j >= t~ - E, where E = err_a |q| sqrt(cmax) + err_b cmax bounds
        // |p~ - p| for this query.  The k-th smallest TRUE value among the kept ones is
        // p_k = delta_k - |q|^2.  If p_k < t~ - E, every reference left out is strictly farther
        // than the k reported: they are the exact answer, ties included.  With no more than krs
        // references in all, nothing was left out.
        const u64 last = keys[kr - 1];
        bool certified = a.all_kept != 0 || last == KEY_INF;
        if (!certified) {
            const float *x = a.Q + q * (int64_t)a.d;
            double qq = 0.0;
            for (int c = lane; c < a.d; c += 64) qq = fma((double)x[c], (double)x[c], qq);
            qq = wave_sum_f64(qq);
            const double cm = (double)*a.cmax;
            const double E = a.err_a * sqrt(qq * cm) + a.err_b * cm;
            const double tt = (double)ord2f((uint32_t)(last >> 32));
            // the reported distance is the double sum rounded to fp32: at most 2^-24 below it
            const double dk = (double)ord2f((uint32_t)(outk[a.k - 1] >> 32)) * (1.0 + 1.2e-7);
            certified = dk - qq < tt - E;
        }
        if (!certified && lane == 0) {
            const int slot = atomicAdd(a.uncert, 1);
            if (a.unc_rows != nullptr && slot < a.unc_cap) a.unc_rows[slot] = (int32_t)q;
        }
    }
}


// The rows a filter pass could not certify, made ready for the fp32 kernel: one wave per row.
__global__ __launch_bounds__(256) void gather_rows(GatherArgs a)
{
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int n = min(*a.count, a.cap);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *a.n_out = n;
        if (a.left_out) *a.left_out = *a.count - n;
    }
    if (i >= n) return;
    const int32_t row = a.rows[i];
    const float *x = a.Q + (int64_t)row * a.d;
    float *o = a.q_out + (int64_t)i * a.dpad;
    for (int c = lane; c < a.dpad; c += 64)
        o[c] = c < a.d ? -2.f * (a.mu != nullptr ? (float)((double)x[c] - (double)a.mu[c]) : x[c]) : 0.f;
    if (lane == 0) {
        a.self_out[i] = a.self_offset >= 0 ? (int32_t)(a.self_offset + row) : -1;
        a.b_out[i] = 0xffffffffu;
    }
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

}  // namespace knn

#endif
