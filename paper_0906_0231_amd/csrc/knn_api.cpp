// Host side of the C ABI declared in include/knn.h: argument checks, workspace
// layout, launch sequence.  No computation happens here.
#include "knn.h"

#include <hip/hip_runtime.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "knn_device.h"

// Workspace of knn_search_static: one array per GPU the library is loaded on, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress; the address
// of a device's copy is looked up once per device (static_scratch()) and that pointer is what
// the kernels receive, exactly as they receive a caller's workspace.
static __device__ __align__(256) unsigned char scratch[KNN_STATIC_SCRATCH_BYTES];

namespace {

using namespace knn;

constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch`; nullptr (and the HIP error in *err) on failure.
void *static_scratch(hipError_t *err)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= MAX_DEVICES)) e = hipErrorInvalidDevice;
    if (e != hipSuccess) { *err = e; return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));     // the copy of the device that is current
        if (e != hipSuccess || !ptr) { *err = e != hipSuccess ? e : hipErrorInvalidSymbol; return nullptr; }
        g_scratch_ptr[dev] = ptr;
    }
    *err = hipSuccess;
    return g_scratch_ptr[dev];
}

thread_local char g_last_error[256] = "";

void set_error(const char *where, hipError_t e)
{
    const char *s = hipGetErrorString(e);
    size_t n = 0;
    for (; where[n] && n < 100; ++n) g_last_error[n] = where[n];
    g_last_error[n++] = ':';
    g_last_error[n++] = ' ';
    for (size_t i = 0; s && s[i] && n < sizeof(g_last_error) - 1; ++i) g_last_error[n++] = s[i];
    g_last_error[n] = 0;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Plan {
    int32_t dpad, kcap, S, n_qtiles, n_rtiles, rt_per_split;
    int64_t nq_pad, n_cpad;
    bool self;      // knn_build: one matrix serves as queries and references
    bool rcopy;     // references need a scaled / padded copy
    bool qreg;      // query tile resident in registers (knn_tiles_qreg)
    bool tri;       // symmetric schedule: rounds of disjoint block pairs (knn_pairs_qreg)
    bool fold;      // distance is not an inner product: vector-ALU kernel (knn_fold)
    bool center;    // squared Euclidean: the references' column means are subtracted from every row first
    size_t off_mu;  // ... [dpad] floats, then [dpad] doubles (the sums they come from)
    bool split;     // split-precision experiment: bf16 pieces, lists of kcap > k entries by approximate value
    int32_t split_waves; // ... waves per workgroup of knn_tiles_split (32 queries each)
    int32_t fb_cap, fb_S, fb_kcap, fb_rt_per_split;   // ... second pass (fp32 kernel) over the rows the filter could
                         //     not certify: most rows it takes, slices, list capacity
    size_t off_fb_q, off_fb_self, off_fb_bound, off_fb_rows, off_fb_words, off_fb_lists, off_r32;
    int64_t refs_per_split; // fold kernel: references per slice, multiple of KNN_FOLD_NR
    bool matrix;    // two-phase organisation: distance matrix written out (knn_dist_qreg), then select_rows
    bool msym;      // ... computing each unordered pair of rows once
    int32_t n_rt64, chunk, n_chunks; // ... reference tiles of 64 rows, tiles per workgroup, workgroups per query tile
    int64_t sel_seg;                 // ... columns per segment of select_rows
    bool mstream;                    // ... d > 256: both operands streamed through LDS (knn_dist_stream)
    bool blocked;                    // ... panel pair by panel pair (the whole matrix would not fit)
    int64_t P;                       // ... rows per panel (multiple of 256)
    size_t off_D2;                   // ... blocked: buffer of the transposed block
    int64_t ldm;                     // ... chunk minima: row pitch in floats, 0 = none
    size_t off_M, off_M2;            // ... [rows of D, ldm] for D and for the transposed block
    bool tau;                        // ... block by block with knn_dist_qreg: chunks above a row's threshold are not stored
    size_t off_tau;                  // ... [nq_pad] value of the k-th entry of every row's list so far
    size_t off_D;                    // ... the matrix, [nq_pad, ldd]; blocked: one block, [P, ldd]
    int64_t ldd;                     // ... its row pitch in floats: n_cpad + 64, an odd multiple of 256 bytes, so that
                                     //     a column of the matrix does not fall into one memory channel
    int32_t B, NB, NBp; // block rows, block count, block count rounded up to even
    int32_t nlists; // partial lists per query
    size_t off_qp, off_rp, off_c, off_sq, off_bound, off_lists, total;
};

int32_t list_capacity(int32_t k)
{
    int32_t c = 16;
    while (c < k) c <<= 1;
    return c;
}

// Split-precision experiment: the lists are kept by approximate value, so they hold more than k
// entries -- a margin of at least two, an eighth of k for long lists -- for the exact re-pricing
// to choose from.
constexpr int32_t KNN_SPLIT_MAX_K = 112;
int32_t split_list_capacity(int32_t k) { return list_capacity(k + (k / 8 > 2 ? k / 8 : 2)); }

// Symmetric schedule: rows per block, and what the schedule costs next to the full square.
// A round is one launch of NBp/2 workgroups, one block pair each, on 512 workgroup slots
// (two per CU), so a round lasts ceil(NBp/2 / 512) pair times whatever its fill; a pair
// costs B*B distance evaluations times (a + c/B), the second term being the sweep's fixed
// part (prologue, mirror hand-over).  a and c are fitted to measured run times at B = 128,
// 256 and 1024 and are larger for long lists, whose mirror merges cost more.  The result is
// the ratio to n*n evaluations spread over the same 512 slots by the full-square kernel;
// B is the multiple of the query tile that minimises it.
double pair_cost_ratio(int64_t n, int32_t B, int32_t kcap)
{
    const int64_t nb = (n + B - 1) / B, nbp = nb + (nb & 1);
    const int64_t pairs = nbp / 2;
    const double a = kcap > 32 ? 1.5 : 1.17, c = kcap > 32 ? 120.0 : 93.0;
    const double rounds = (double)(nbp - 1) * (double)((pairs + 511) / 512) + (double)((nb + 511) / 512);  // + the diagonal blocks
    return 512.0 * rounds * (double)B * (double)B * (a + c / (double)B) / ((double)n * (double)n);
}

int32_t pair_block_rows(int64_t n, int32_t kcap)
{
    int32_t best = KNN_TILE;
    double best_ratio = pair_cost_ratio(n, best, kcap);
    for (int32_t b = 2 * KNN_TILE; b <= 8192 && b < 2 * n; b += KNN_TILE) {
        const double r = pair_cost_ratio(n, b, kcap);
        if (r < best_ratio - 1e-12) { best_ratio = r; best = b; }
    }
    return best;
}

// knn_select: how the columns are cut.  Enough waves to fill the GPU when there are few rows,
// segments no shorter than 16K columns, and no more partial lists than finalize can merge.
void select_plan(int64_t m, int64_t n, int32_t k, int32_t &kcap, int32_t &S, int64_t &seg)
{
    kcap = list_capacity(k);
    int64_t want = (4096 + m - 1) / m;       // waves wanted in all; measured: more (shorter) segments only add lists
    int64_t most = n / 16384 > 0 ? n / 16384 : 1;
    if (want > most) want = most;
    if (want > KNN_FIN_MAX / kcap) want = KNN_FIN_MAX / kcap;
    if (want < 1) want = 1;
    seg = (n + want - 1) / want;
    seg = (seg + 1023) / 1024 * 1024;
    S = (int32_t)((n + seg - 1) / seg);
}

// Two-phase plan: is the matrix written out whole or block by block, and with which panel size.
// Whole while it is at most 72 GiB.  Beyond that, for knn_build with a symmetric distance, the
// rows are cut into panels of 65 536 (two block buffers of 17 GB) and every pair of panels is
// written once; block_rows > 0 with variant 4 sets the panel size and forces this form at any
// size (tests).  Returns false if the two-phase plan cannot be used at all.
constexpr double KNN_MATRIX_CAP_BYTES = 72.0 * 1073741824.0;
bool two_phase_layout(Plan &p, int64_t cpad128, double matrix_bytes, bool msym, int32_t variant, int32_t block_rows)
{
    p.blocked = false;
    p.P = 0;
    int64_t P = 65536;
    const bool forced = variant == 4 && block_rows > 0 && msym;
    if (forced) P = (int64_t)align_up((size_t)block_rows, 256);
    if ((forced || matrix_bytes > KNN_MATRIX_CAP_BYTES) && P < cpad128) {
        if (!msym) return false;                  // no pair of rows to save: the fused kernels do that better
        p.blocked = true;
        p.P = P;
        p.ldd = P + 64;
    }
    return true;
}

// Sizes are assumed validated.  r_splits == 0 picks the slice count of the reference range
// (see below), block_rows == 0 and symmetric == 0 take the cost model above.
bool make_plan_core(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric, bool self,
                    int32_t r_splits, int32_t variant, int32_t symmetric, int32_t block_rows, bool center, Plan &p)
{
    p.self = self;
    p.center = center;
    p.split = false;
    p.split_waves = 0;
    p.fold = metric == KNN_L1 || metric == KNN_LINF;
    p.refs_per_split = 0;
    p.matrix = p.msym = false;
    p.n_rt64 = p.chunk = p.n_chunks = 0;
    p.sel_seg = 0;
    p.off_D = p.off_D2 = 0;
    p.off_M = p.off_M2 = 0;
    p.ldm = 0;
    p.tau = false;
    p.off_tau = 0;
    p.ldd = 0;
    p.blocked = false;
    p.mstream = false;
    p.P = 0;
    if (p.fold) {
        // lane = query, 64 per wave; the reference range is cut so that the device has
        // several thousand waves to run
        p.dpad = (int32_t)align_up((size_t)d, 4);
        p.qreg = p.tri = false;
        p.rcopy = true;
        p.kcap = list_capacity(k);
        p.n_qtiles = (int32_t)((nq + KNN_TILE - 1) / KNN_TILE);
        p.n_rtiles = (int32_t)((nr + KNN_TILE - 1) / KNN_TILE);
        p.nq_pad = (int64_t)p.n_qtiles * KNN_TILE;
        p.n_cpad = (nr + KNN_FOLD_NR - 1) / KNN_FOLD_NR * KNN_FOLD_NR;
        p.B = p.NB = p.NBp = 0;
        // Two-phase form of the fold (distances written out, then select_rows): on request, or by
        // default while the matrix is at most 72 GiB for long lists, for knn_build with d >= 64,
        // where computing each pair once halves the vector work that bounds this path (measured:
        // n = 65 536, d = 128, k = 32 28.0 -> 18.2 ms; d = 64 13.5 -> 11.7 ms), and for small
        // problems (n = 16 384: 4.0 -> 1.5 ms).
        {
            const int64_t cpad128 = (nr + KNN_TILE - 1) / KNN_TILE * KNN_TILE;
            p.ldd = cpad128 + 64;
            const double matrix_bytes = (double)p.nq_pad * (double)p.ldd * sizeof(float);
            const bool msym = self && symmetric != 2;
            const bool matrix_ok = cpad128 < ((int64_t)1 << 28);
            if (variant == 4)
                p.matrix = matrix_ok;
            else if (variant == 0 && matrix_ok && matrix_bytes <= KNN_MATRIX_CAP_BYTES)
                p.matrix = p.kcap > 32 || (msym ? d >= 64 : matrix_bytes <= 4.0 * 1073741824.0);
            else if (variant == 0 && matrix_ok)
                p.matrix = msym && d >= 64;       // blocked: half the vector work at any size
            if (p.matrix) p.matrix = two_phase_layout(p, cpad128, matrix_bytes, msym, variant, block_rows);
            if (p.matrix) {
                p.msym = msym;
                p.n_rt64 = (int32_t)((nr + KNN_FOLD_NR - 1) / KNN_FOLD_NR);
                const int64_t qblocks = (nq + 255) / 256;
                const int64_t tiles = p.blocked ? (p.P / 256) * (p.P / KNN_FOLD_NR) : qblocks * p.n_rt64 / (p.msym ? 2 : 1);
                int64_t chunk = (tiles + 2047) / 2048;     // 4 workgroups fit a CU: aim at two rounds of them
                if (chunk < 4) chunk = 4;
                if (chunk > 64) chunk = 64;
                p.chunk = (int32_t)chunk;
                p.n_chunks = (p.n_rt64 + p.chunk - 1) / p.chunk;
                int32_t skcap;
                select_plan(nq, nr, k, skcap, p.S, p.sel_seg);
                if (p.blocked) p.S = 1;
                p.nlists = p.S;
                p.rt_per_split = 0;
                size_t o = 0;
                p.off_qp = o;
                o = align_up(o + (size_t)p.nq_pad * p.dpad * sizeof(float), 256);
                p.off_rp = o;
                o = align_up(o + (size_t)p.n_cpad * p.dpad * sizeof(float), 256) + 256;
                p.off_c = p.off_sq = p.off_bound = o;
                p.off_D = o;
                o = align_up(o + (size_t)(p.blocked ? p.P : p.nq_pad) * p.ldd * sizeof(float), 256);
                p.off_D2 = o;
                if (p.blocked) o = align_up(o + (size_t)p.P * p.ldd * sizeof(float), 256);
                p.ldm = (p.ldd / 32 + 15) / 16 * 16;  // minimum of every chunk of 32 columns, for select_rows_sparse
                p.off_M = o;
                o = align_up(o + (size_t)(p.blocked ? p.P : p.nq_pad) * p.ldm * sizeof(float), 256);
                p.off_M2 = o;
                if (p.blocked) o = align_up(o + (size_t)p.P * p.ldm * sizeof(float), 256);
                p.off_lists = o;
                o = align_up(o + (size_t)p.nlists * nq * p.kcap * sizeof(u64), 256);
                p.total = o;
                return true;
            }
        }
        const int64_t groups = (nq + 63) / 64;
        int64_t S = r_splits > 0 ? r_splits : (8192 + groups - 1) / groups;
        const int64_t smax = KNN_FIN_MAX / p.kcap;
        if (S > smax) S = smax;
        if (S < 1) S = 1;
        p.refs_per_split = (int64_t)align_up((size_t)((nr + S - 1) / S), KNN_FOLD_NR);
        p.S = (int32_t)((nr + p.refs_per_split - 1) / p.refs_per_split);
        p.rt_per_split = 0;
        p.nlists = p.S;
        size_t o = 0;
        p.off_qp = o;                                 // queries packed by tile of 64 rows
        o = align_up(o + (size_t)p.nq_pad * p.dpad * sizeof(float), 256);
        p.off_rp = o;                                 // references packed by tile
        o = align_up(o + (size_t)p.n_cpad * p.dpad * sizeof(float), 256) + 256;   // + one batch of read-ahead
        p.off_c = o;                                  // here: one bound word per query
        o = align_up(o + (size_t)p.nq_pad * sizeof(uint32_t), 256);
        p.off_sq = o;
        p.off_bound = o;
        p.off_lists = o;
        o = align_up(o + (size_t)p.nlists * p.nq_pad * p.kcap * sizeof(u64), 256);
        p.total = o;
        return true;
    }
    if (variant == KNN_PLAN_SPLIT_BF16) {
        // fused full square on the bf16 matrix instructions; the caller has checked metric, d and k
        p.split = true;
        p.split_waves = 8;
        p.dpad = (int32_t)align_up((size_t)d, 32);
        p.qreg = true;
        p.rcopy = true;
        p.kcap = split_list_capacity(k);
        // each pair once (the tournament of knn_pairs_qreg, which works on tiles of 128 queries): on
        // request only.  With products this cheap the mirror update costs what the halved products
        // save: n = 2^20, d = 256: 1421 ms against 1341 ms for the full square; n = 65 536, d = 128,
        // k = 32: 24.7 against 9.8 ms.
        p.B = block_rows > 0 ? (int32_t)align_up((size_t)block_rows, KNN_TILE) : pair_block_rows(nr, p.kcap);
        p.tri = self && symmetric == 1;
        p.NB = (int32_t)((nr + p.B - 1) / p.B);
        p.NBp = p.NB + (p.NB & 1);
        const int32_t tq = p.tri ? KNN_TILE : 32 * p.split_waves;
        p.n_qtiles = (int32_t)((nq + tq - 1) / tq);
        p.n_rtiles = (int32_t)((nr + KNN_TILE - 1) / KNN_TILE);
        p.nq_pad = (int64_t)p.n_qtiles * tq;
        p.n_cpad = (int64_t)p.n_rtiles * KNN_TILE;
        // slices of the reference range as for the fp32 kernel
        int32_t smax = KNN_FIN_MAX / p.kcap;
        if (smax > p.n_rtiles) smax = p.n_rtiles;
        int32_t S = r_splits;
        if (S <= 0) {
            const int32_t slots = 2048 / p.split_waves;          // workgroups the device holds at once
            const int32_t cap = (p.n_qtiles >= slots && p.kcap > 32) ? 1 : (4 * slots + p.n_qtiles - 1) / p.n_qtiles;
            double best = -1.0;
            S = 1;
            for (int32_t s = 1; s <= cap && s <= smax; ++s) {
                const int64_t wg = (int64_t)p.n_qtiles * s;
                const double eff = (double)wg / (double)((wg + slots - 1) / slots * slots);
                if (eff >= 0.9) { S = s; break; }
                if (eff > best + 1e-9) { best = eff; S = s; }
            }
        }
        if (S > smax) S = smax;
        if (S < 1) S = 1;
        if (p.tri) S = 1;
        p.rt_per_split = (p.n_rtiles + S - 1) / S;
        p.S = (p.n_rtiles + p.rt_per_split - 1) / p.rt_per_split;
        p.nlists = p.S;
        size_t o = 0;
        p.off_qp = o;
        o = align_up(o + (size_t)nq * p.dpad * sizeof(float), 256);
        p.off_rp = o;
        o = align_up(o + (size_t)nr * p.dpad * sizeof(float), 256);
        p.off_c = o;
        o = align_up(o + (size_t)p.n_cpad * sizeof(float), 256);
        p.off_sq = o;
        o = align_up(o + (size_t)nq * sizeof(float), 256) + 256;   // + one scalar (max c_j)
        p.off_bound = o;
        o = align_up(o + (size_t)nq * sizeof(uint32_t), 256);
        p.off_lists = o;
        o = align_up(o + (size_t)p.nlists * p.nq_pad * p.kcap * sizeof(u64), 256);
        // second pass: at most 4096 rows, the reference range in as many slices as finalize can merge
        p.fb_cap = (int32_t)(nq < 4096 ? (nq + KNN_TILE - 1) / KNN_TILE * KNN_TILE : 4096);
        p.fb_kcap = list_capacity(k);
        int32_t s2 = KNN_FIN_MAX / p.fb_kcap;
        if (s2 > p.n_rtiles) s2 = p.n_rtiles;
        p.fb_rt_per_split = (p.n_rtiles + s2 - 1) / s2;
        p.fb_S = (p.n_rtiles + p.fb_rt_per_split - 1) / p.fb_rt_per_split;
        p.off_fb_q = o;
        o = align_up(o + (size_t)p.fb_cap * p.dpad * sizeof(float), 256);
        p.off_fb_self = o;
        o = align_up(o + (size_t)p.fb_cap * sizeof(int32_t), 256);
        p.off_fb_bound = o;
        o = align_up(o + (size_t)p.fb_cap * sizeof(uint32_t), 256);
        p.off_fb_rows = o;
        o = align_up(o + (size_t)p.fb_cap * sizeof(int32_t), 256);
        p.off_fb_words = o;                        // [0] rows not certified by the first pass, [1] rows in the second
        o += 256;
        p.off_fb_lists = o;
        o = align_up(o + (size_t)p.fb_S * p.fb_cap * p.fb_kcap * sizeof(u64), 256);
        p.off_r32 = o;                             // fp32 reference rows padded to dpad (and centred), if d is ragged (or centred)
        if (p.dpad != d || p.center) o = align_up(o + (size_t)nr * p.dpad * sizeof(float), 256);
        p.total = o;
        return true;
    }
    p.dpad = (int32_t)align_up((size_t)d, KNN_DC);
    const int32_t dpad32 = (int32_t)align_up((size_t)d, 32);
    p.qreg = (variant == 0 || variant == 3) && dpad32 <= KNN_QRES_MAX_D;
    if (p.qreg) p.dpad = dpad32;
    p.kcap = list_capacity(k);
    p.n_qtiles = (int32_t)((nq + KNN_TILE - 1) / KNN_TILE);
    p.n_rtiles = (int32_t)((nr + KNN_TILE - 1) / KNN_TILE);
    p.nq_pad = (int64_t)p.n_qtiles * KNN_TILE;
    p.n_cpad = (int64_t)p.n_rtiles * KNN_TILE;
    // symmetric schedule: only for knn_build, only with the register-resident kernel;
    // by default only where the cost model puts it below the full square
    p.B = block_rows > 0 ? (int32_t)align_up((size_t)block_rows, KNN_TILE) : pair_block_rows(nr, p.kcap);
    p.tri = self && p.qreg && metric != KNN_KL && symmetric != 2 &&
            (symmetric == 1 || (nr >= 512 * KNN_TILE && pair_cost_ratio(nr, p.B, p.kcap) < 0.97));
    p.NB = (int32_t)((nr + p.B - 1) / p.B);
    p.NBp = p.NB + (p.NB & 1);
    // Two-phase organisation (matrix written out, then selected from): on request, or by default
    // where it was measured faster than the fused kernels and the matrix is at most 72 GiB:
    // long lists (the fused kernels then spend more time merging candidates than multiplying:
    // 2 to 3 times faster on the shapes of the paper's Table 1); knn_build with d >= 128, where
    // computing each pair once saves more than the matrix costs to write and read back (below
    // that the stores bound it: 4 n^2 bytes against n^2 d flop); and small problems, which its
    // two-dimensional grid spreads over the device better than one sweep per query tile does.
    // d <= 256 uses the register-resident operand layout (knn_dist_qreg), larger d the streaming one.
    p.ldd = p.n_cpad + 64;
    const double matrix_bytes = (double)p.nq_pad * (double)p.ldd * sizeof(float);
    const bool matrix_ok = p.n_cpad < ((int64_t)1 << 28);   // 32-bit element offsets within four rows
    const bool msym = self && metric != KNN_KL && symmetric != 2;
    p.matrix = false;
    if (variant == 4)
        p.matrix = matrix_ok;
    else if (variant == 0 && symmetric != 1 && matrix_ok && matrix_bytes <= KNN_MATRIX_CAP_BYTES)
        p.matrix = p.kcap > 32 || (msym ? (dpad32 >= 128 || p.n_cpad <= 49152) : matrix_bytes <= 4.0 * 1073741824.0);
    else if (variant == 0 && symmetric != 1 && matrix_ok)
        // block by block, for d > 96 (below that the stores of the first sweep and the minima
        // bound it: d = 64, n = 262 144, k = 100: 100 ms against 108).  Measured, ms fused ->
        // blocked, k = 10: d = 256: n = 150 000 99 -> 65, 262 144 197 -> 149, 524 288 688 -> 572,
        // 2^20 2457 -> 2254; d = 128: n = 262 144 101 -> 88, 524 288 343 -> 337, 2^20 1281 -> 1308
        // (k = 32: 1409 -> 1356); k = 100, d = 256: n = 262 144 293 -> 156, 2^20 3201 -> 2700.
        p.matrix = msym && dpad32 >= 128;
    if (p.matrix) p.matrix = two_phase_layout(p, p.n_cpad, matrix_bytes, msym, variant, block_rows);
    if (p.matrix) {
        p.mstream = dpad32 > KNN_QRES_MAX_D;       // p.dpad stays d rounded up to KNN_DC then
        if (!p.mstream) p.dpad = dpad32;
        p.qreg = p.tri = false;
        p.msym = msym;
        const int32_t tr = p.mstream ? KNN_TILE : 64;              // reference rows per tile of the distance kernel
        p.n_rt64 = (int32_t)((nr + tr - 1) / tr);
        const int64_t tiles = p.blocked ? (p.P / KNN_TILE) * (p.P / tr)
                                        : (int64_t)p.n_qtiles * p.n_rt64 / (p.msym ? 2 : 1);
        int64_t chunk = (tiles + 1023) / 1024;
        if (chunk < (p.mstream ? 2 : 4)) chunk = p.mstream ? 2 : 4;
        if (chunk > (p.mstream ? 32 : 64)) chunk = p.mstream ? 32 : 64;
        if (!p.mstream && !p.blocked && tiles >= 8192) {
            // whole matrix, d <= 256, enough tiles to go round: about six workgroups per slot (512 slots) even out the unequal
            // sweeps of the triangle, but no fewer than 8 tiles each, which is what a workgroup's
            // start (query operands into registers) wants to be spread over.  Measured, ms of the
            // distance kernel with 1024 workgroups in all -> this rule: n = 20 000, d = 256: 1.13 ->
            // 0.99; 40 000: 4.09 -> 3.62; 80 000: 14.19 -> 14.04; 65 536, d = 128: 6.41 -> 6.20.
            chunk = (tiles + 3071) / 3072;
            if (chunk < 8) chunk = 8;
            if (chunk > 48) chunk = 48;
        }
        p.chunk = (int32_t)chunk;
        p.n_chunks = (p.n_rt64 + p.chunk - 1) / p.chunk;
        int32_t skcap;
        select_plan(nq, nr, k, skcap, p.S, p.sel_seg);
        if (p.blocked) p.S = 1;                   // lists are continued from block to block: one per row
        p.nlists = p.S;
        p.rt_per_split = 0;
        p.rcopy = metric != KNN_SQEUCLIDEAN || p.dpad != d || p.center;
        size_t o = 0;
        p.off_qp = o;
        o = align_up(o + (size_t)nq * p.dpad * sizeof(float), 256);
        p.off_rp = o;
        if (p.rcopy) o = align_up(o + (size_t)nr * p.dpad * sizeof(float), 256);
        p.off_c = o;
        o = align_up(o + (size_t)p.n_cpad * sizeof(float), 256);
        p.off_sq = o;
        o = align_up(o + (size_t)nq * sizeof(float), 256) + 256;
        p.off_bound = o;
        p.off_D = o;
        o = align_up(o + (size_t)(p.blocked ? p.P : p.nq_pad) * p.ldd * sizeof(float), 256);
        p.off_D2 = o;
        if (p.blocked) o = align_up(o + (size_t)p.P * p.ldd * sizeof(float), 256);
        {
            // minimum of every chunk of 32 columns, so that select_rows can skip most of a row
            p.ldm = (p.ldd / 32 + 15) / 16 * 16;
            p.off_M = o;
            o = align_up(o + (size_t)(p.blocked ? p.P : p.nq_pad) * p.ldm * sizeof(float), 256);
            p.off_M2 = o;
            if (p.blocked) o = align_up(o + (size_t)p.P * p.ldm * sizeof(float), 256);
            p.tau = p.blocked;
            p.off_tau = o;
            if (p.tau) o = align_up(o + (size_t)p.nq_pad * sizeof(float), 256);
        }
        p.off_lists = o;
        o = align_up(o + (size_t)p.nlists * nq * p.kcap * sizeof(u64), 256);
        p.total = o;
        return true;
    }
    int32_t smax = KNN_FIN_MAX / p.kcap;
    if (smax > p.n_rtiles) smax = p.n_rtiles;
    int32_t S = r_splits;
    if (S <= 0) {
        // The device holds 512 workgroups of the tile kernels at once (two per CU).  With fewer
        // query tiles than that, take the smallest slice count that fills at least 90 % of the
        // last round of workgroups (every slice costs each query a list of its own: k forced
        // insertions and a merge at the end), else the one that fills it best.  With more tiles
        // than that and long lists, one slice: measured faster even when the second round of
        // workgroups is short (n = 80 000, k = 100), while with short lists balancing the second
        // round still pays (n = 100 000, k = 10).
        const int32_t cap = (p.n_qtiles >= 512 && p.kcap > 32) ? 1 : (2048 + p.n_qtiles - 1) / p.n_qtiles;
        double best = -1.0;
        S = 1;
        for (int32_t s = 1; s <= cap && s <= smax; ++s) {
            const int64_t wg = (int64_t)p.n_qtiles * s;
            const double eff = (double)wg / (double)((wg + 511) / 512 * 512);
            if (eff >= 0.9) {
                S = s;
                break;
            }
            if (eff > best + 1e-9) {
                best = eff;
                S = s;
            }
        }
    }
    if (S > smax) S = smax;
    if (S < 1) S = 1;
    if (p.tri) S = 1;
    p.rt_per_split = (p.n_rtiles + S - 1) / S;
    p.S = (p.n_rtiles + p.rt_per_split - 1) / p.rt_per_split;
    p.nlists = p.S;
    p.rcopy = metric != KNN_SQEUCLIDEAN || p.dpad != d || p.center;

    size_t o = 0;
    p.off_qp = o;
    o = align_up(o + (size_t)nq * p.dpad * sizeof(float), 256);
    p.off_rp = o;
    if (p.rcopy) o = align_up(o + (size_t)nr * p.dpad * sizeof(float), 256);
    p.off_c = o;
    o = align_up(o + (size_t)p.n_cpad * sizeof(float), 256);
    p.off_sq = o;
    o = align_up(o + (size_t)nq * sizeof(float), 256) + 256;   // + one scalar (max c_j)
    p.off_bound = o;                                 // one word per query: bound shared by the slices
    o = align_up(o + (size_t)nq * sizeof(uint32_t), 256);
    p.off_lists = o;
    o = align_up(o + (size_t)p.nlists * p.nq_pad * p.kcap * sizeof(u64), 256);
    p.total = o;
    return true;
}

// knn_options_t.center applies to the squared Euclidean distance only (a translation changes the
// cosine and correlation distances, and the others do not go through the expanded form); the
// means and their sums follow whatever the plan itself needs.
bool make_plan(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric, bool self,
               int32_t r_splits, int32_t variant, int32_t symmetric, int32_t block_rows, int32_t center, Plan &p)
{
    const bool ok = make_plan_core(nq, nr, d, k, metric, self, r_splits, variant, symmetric, block_rows,
                                   center == 1 && metric == KNN_SQEUCLIDEAN, p);
    p.off_mu = p.total;
    if (p.center) p.total += align_up((size_t)p.dpad * sizeof(float), 256) + align_up((size_t)p.dpad * sizeof(double), 256);
    return ok;
}

knn_status_t check_sizes(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric,
                         int64_t self_offset)
{
    if (nq < 1 || nr < 1 || d < 1 || k < 1) return KNN_EINVAL;
    if ((int)metric < (int)KNN_SQEUCLIDEAN || (int)metric > (int)KNN_KL) return KNN_EINVAL;
    if (self_offset < -1) return KNN_EINVAL;
    if (self_offset >= 0 && self_offset + nq > nr) return KNN_EINVAL;
    if ((int64_t)k > nr - (self_offset >= 0 ? 1 : 0)) return KNN_EINVAL;
    if (nr >= ((int64_t)1 << 31) || nq >= ((int64_t)1 << 31)) return KNN_EUNSUPPORTED;
    if (d > (1 << 20)) return KNN_EUNSUPPORTED;
    if (k > KNN_MAX_K) return KNN_EUNSUPPORTED;
    return KNN_OK;
}


knn_status_t check_options(const knn_options_t &o)
{
    if (o.symmetric < 0 || o.symmetric > 2 || o.rescore < 0 || o.rescore > 2 || o.r_splits < 0 ||
        o.block_rows < 0 || o.block_rows > (1 << 20) || o.center < 0 || o.center > 1)
        return KNN_EINVAL;
    if (o.variant != KNN_PLAN_AUTO && o.variant != KNN_PLAN_FUSED_STREAMING && o.variant != KNN_PLAN_FUSED &&
        o.variant != KNN_PLAN_TWO_PHASE && o.variant != KNN_PLAN_SPLIT_BF16)
        return KNN_EINVAL;
    return KNN_OK;
}

// what the split-precision plan can serve
knn_status_t check_split(const knn_options_t &o, int32_t d, int32_t k, knn_metric_t metric)
{
    if (o.variant != KNN_PLAN_SPLIT_BF16) return KNN_OK;
    if (metric != KNN_SQEUCLIDEAN || d > KNN_QRES_MAX_D || k > KNN_SPLIT_MAX_K) return KNN_EUNSUPPORTED;
    return KNN_OK;
}

// The plan of a call.  A plan named in the options is taken as such.  KNN_PLAN_AUTO takes the
// preferred plan (make_plan's choice, which may keep distances in the workspace) if it fits in
// `budget` bytes, else the fused plan, which needs only copies of the inputs and the lists.
// KNN_ENOMEM if even that does not fit.  Sizes and options are assumed validated.
knn_status_t choose_plan(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric, bool self,
                         const knn_options_t &o, size_t budget, Plan &p)
{
    make_plan(nq, nr, d, k, metric, self, o.r_splits, o.variant, o.symmetric, o.block_rows, o.center, p);
    if (p.total <= budget) return KNN_OK;
    if (o.variant != KNN_PLAN_AUTO || !p.matrix) return KNN_ENOMEM;
    make_plan(nq, nr, d, k, metric, self, o.r_splits, KNN_PLAN_FUSED, o.symmetric, o.block_rows, o.center, p);
    return p.total <= budget ? KNN_OK : KNN_ENOMEM;
}

// kernel launches of the distance + selection stage
int32_t plan_launches(const Plan &p, int64_t nr)
{
    if (p.matrix && p.blocked) {
        const int64_t G = (nr + p.P - 1) / p.P;
        return (int32_t)(G * (G + 1) / 2 + G * G);          // one block per panel pair, one selection per block and side
    }
    if (p.matrix) return 2;
    if (p.tri) return p.NBp;                                // the diagonal blocks, then NBp - 1 rounds
    return 1;
}

const char *plan_kernel(const Plan &p)
{
    if (p.split) return p.tri ? "knn_pairs_qreg" : "knn_tiles_split";
    if (p.fold) return p.matrix ? "knn_fold_dist" : "knn_fold";
    if (p.matrix) return p.mstream ? "knn_dist_stream" : "knn_dist_qreg";
    if (p.tri) return "knn_pairs_qreg";
    return p.qreg ? "knn_tiles_qreg" : "knn_tiles";
}

struct Events {
    hipEvent_t e[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    std::vector<hipEvent_t> span;    // pairs (before, after) around the launches of one kind, see bracket()
    bool on = false;
    hipError_t create()
    {
        for (auto &x : e) {
            hipError_t r = hipEventCreate(&x);
            if (r != hipSuccess) return r;
        }
        on = true;
        return hipSuccess;
    }
    void record(int i, hipStream_t s)
    {
        if (on) (void)hipEventRecord(e[i], s);
    }
    // one more event on the stream, kept in `span` (profiling only; a failure just drops it)
    void bracket(hipStream_t s)
    {
        if (!on) return;
        hipEvent_t x = nullptr;
        if (hipEventCreate(&x) != hipSuccess) return;
        (void)hipEventRecord(x, s);
        span.push_back(x);
    }
    // sum over the pairs, once the stream has been waited for
    float bracketed_ms() const
    {
        float sum = 0.f;
        for (size_t i = 0; i + 1 < span.size(); i += 2) {
            float t = 0.f;
            if (hipEventElapsedTime(&t, span[i], span[i + 1]) == hipSuccess) sum += t;
        }
        return sum;
    }
    ~Events()
    {
        for (auto &x : e)
            if (x) (void)hipEventDestroy(x);
        for (auto &x : span) (void)hipEventDestroy(x);
    }
};

// Phase 1 + Phase 2 of the two-phase plan.  Whole matrix: one launch of the distance kernel
// (all of it, or the triangle mirrored) and one of select_rows.  Blocked (the matrix would not
// fit): the rows are cut into panels of p.P; for every unordered pair of panels (a, b) the block
// D[a][b] is written once, together with its transpose if a != b, and select_rows continues the
// lists of the rows of a (and of b) with the columns of that block.
knn_status_t run_two_phase(const Plan &p, const float *Q, int64_t nq, const float *R, int64_t nr, int32_t d,
                           int32_t k, knn_metric_t metric, int64_t self_offset, float *qp, float *rp, float *cr,
                           u64 *lists, char *ws, hipStream_t stream, Events &ev, int32_t &launches,
                           int64_t &pairs_computed)
{
    (void)Q;
    float *D0 = (float *)(ws + p.off_D);
    float *D1 = (float *)(ws + p.off_D2);
    float *M0 = p.ldm ? (float *)(ws + p.off_M) : nullptr;
    float *M1 = p.ldm ? (float *)(ws + p.off_M2) : nullptr;
    launches = 0;
    pairs_computed = 0;
    hipError_t e;

    // one block: queries [q0, q0 + mq) against references [r0, r0 + mr)
    // full_q / full_r: the query rows / the rows the mirrored values go to have been through select_rows (p.tau only)
    float *tau = p.tau ? (float *)(ws + p.off_tau) : nullptr;
    auto dist = [&](int64_t q0, int64_t mq, int64_t r0, int64_t mr, int mode, int64_t self_off, bool full_q,
                    bool full_r) -> hipError_t {
        ++launches;
        if (p.fold) {
            FoldDistArgs fd;
            fd.Qpk = qp + q0 * p.dpad;              // packed by tiles of 64 rows; q0 is a multiple of 256
            fd.Rpk = rp + r0 * p.dpad;
            fd.D = D0;
            fd.Dm = mode == DIST_RECT_MIRROR ? D1 : D0;
            fd.M = M0;
            fd.Mm = mode == DIST_RECT_MIRROR ? M1 : M0;
            fd.ldm = p.ldm;
            fd.ldd = p.ldd;
            fd.nq = mq;
            fd.nr = mr;
            fd.self_offset = self_off;
            fd.n_tiles = (mr + KNN_FOLD_NR - 1) / KNN_FOLD_NR;
            fd.dpad = p.dpad;
            fd.metric = (int32_t)metric;
            fd.chunk = p.chunk;
            fd.n_chunks = (int32_t)((fd.n_tiles + p.chunk - 1) / p.chunk);
            fd.n_qblocks = (int32_t)((mq + 255) / 256);
            const int64_t groups = (mq + 63) / 64;
            if (mode == DIST_TRIANGLE) {
                for (int64_t g = 0; g < groups; ++g)
                    if (fd.n_tiles > g) pairs_computed += (fd.n_tiles - g) * 64 * KNN_FOLD_NR;
            } else {
                pairs_computed += groups * 64 * fd.n_tiles * KNN_FOLD_NR;
            }
            return launch_fold_dist(fd, mode, stream);
        }
        DistArgs da;
        da.Qp = qp + q0 * p.dpad;
        da.ldq = p.dpad;
        da.ldr = p.rcopy ? p.dpad : d;
        da.Rp = (p.rcopy ? rp : R) + r0 * da.ldr;
        da.cR = cr + r0;
        da.cQ = cr + q0;                           // read when values are mirrored: queries are rows of the same set
        da.D = D0;
        da.Dm = mode == DIST_RECT_MIRROR ? D1 : D0;
        da.M = M0;
        da.Mm = mode == DIST_RECT_MIRROR ? M1 : M0;
        da.tauQ = tau && full_q && M0 ? tau + q0 : nullptr;
        da.tauR = tau && full_r && M0 ? tau + r0 : nullptr;
        da.ldm = p.ldm;
        da.ldd = p.ldd;
        da.nq = mq;
        da.nr = mr;
        da.self_offset = self_off;
        da.dpad = p.dpad;
        const int32_t tr = p.mstream ? KNN_TILE : 64;              // reference rows per tile
        da.n_rt = (int32_t)((mr + tr - 1) / tr);
        da.chunk = p.chunk;
        da.n_chunks = (da.n_rt + p.chunk - 1) / p.chunk;
        da.n_qtiles = (int32_t)((mq + KNN_TILE - 1) / KNN_TILE);
        const int32_t per_q = KNN_TILE / tr;                       // reference tiles per query tile
        if (mode == DIST_TRIANGLE) {
            for (int32_t qt = 0; qt < da.n_qtiles; ++qt)
                if (da.n_rt > per_q * qt) pairs_computed += (int64_t)(da.n_rt - per_q * qt) * KNN_TILE * tr;
        } else {
            pairs_computed += (int64_t)da.n_qtiles * KNN_TILE * da.n_rt * tr;
        }
        return p.mstream ? launch_dist_stream(da, da.n_qtiles, mode, stream)
                         : launch_dist_qreg(da, da.n_qtiles, mode, stream);
    };
    auto select = [&](const float *A, int64_t row0, int64_t m, int64_t col0, int64_t ncols, int32_t S, int64_t seg,
                      bool resume) -> hipError_t {
        ++launches;
        SelectArgs sa;
        sa.A = A;
        sa.lists = lists + row0 * p.kcap;
        sa.m = m;
        sa.n = ncols;
        sa.lda = p.ldd;
        sa.seg = seg;
        sa.k = k;
        sa.kcap = p.kcap;
        sa.S = S;
        sa.vec4 = 1;                               // rows of the matrix start on 256-byte boundaries
        sa.resume = resume ? 1 : 0;
        sa.col0 = col0;
        sa.M = A == D0 ? M0 : M1;
        sa.ldm = p.ldm;
        sa.tau_out = tau && S == 1 ? tau + row0 : nullptr;
        return launch_select(sa, stream);
    };

    if (!p.blocked) {
        e = dist(0, nq, 0, nr, p.msym ? DIST_TRIANGLE : DIST_FULL, self_offset, false, false);
        if (e != hipSuccess) { set_error(p.fold ? "knn_fold_dist" : p.mstream ? "knn_dist_stream" : "knn_dist_qreg", e); return KNN_EDEVICE; }
        ev.record(4, stream);
        e = select(D0, 0, nq, 0, nr, p.S, p.sel_seg, false);
        if (e != hipSuccess) { set_error("select_rows", e); return KNN_EDEVICE; }
        return KNN_OK;
    }
    // panel pairs; one list per row, continued from block to block (one wave per row: a block's
    // row segment is at most p.P columns)
    const int64_t G = (nr + p.P - 1) / p.P;
    const int64_t seg = (p.P + 1023) / 1024 * 1024;
    for (int64_t a = 0; a < G; ++a) {
        const int64_t q0 = a * p.P, mq = nr - q0 < p.P ? nr - q0 : p.P;
        for (int64_t b = a; b < G; ++b) {
            const int64_t r0 = b * p.P, mr = nr - r0 < p.P ? nr - r0 : p.P;
            // rows of panel a were first seen in block (0, a) (mirrored) or, for a = 0, right here
            const bool seen_a = !(a == 0 && b == 0), seen_b = a != 0;
            ev.bracket(stream);
            e = dist(q0, mq, r0, mr, a == b ? DIST_TRIANGLE : DIST_RECT_MIRROR, a == b ? 0 : -1, seen_a, seen_b);
            ev.bracket(stream);
            if (e != hipSuccess) { set_error(p.fold ? "knn_fold_dist" : p.mstream ? "knn_dist_stream" : "knn_dist_qreg", e); return KNN_EDEVICE; }
            e = select(D0, q0, mq, r0, mr, 1, seg, seen_a);
            if (e != hipSuccess) { set_error("select_rows", e); return KNN_EDEVICE; }
            if (a != b) {
                e = select(D1, r0, mr, q0, mq, 1, seg, seen_b);
                if (e != hipSuccess) { set_error("select_rows", e); return KNN_EDEVICE; }
            }
        }
    }
    return KNN_OK;
}

knn_status_t run(const float *Q, int64_t nq, const float *R, int64_t nr, int32_t d, int32_t k,
                 knn_metric_t metric, int64_t self_offset, bool self, int32_t *idx, float *dist,
                 void *workspace, size_t workspace_bytes, void *stream_v, const knn_options_t *opt)
{
    g_last_error[0] = 0;
    if (!Q || !R || !idx || !dist) return KNN_EINVAL;
    knn_status_t st = check_sizes(nq, nr, d, k, metric, self_offset);
    if (st != KNN_OK) return st;
    if (((uintptr_t)Q & 15) || ((uintptr_t)R & 15) || ((uintptr_t)idx & 3) || ((uintptr_t)dist & 3))
        return KNN_EINVAL;
    knn_options_t o;
    memset(&o, 0, sizeof(o));
    if (opt) o = *opt;
    st = check_options(o);
    if (st == KNN_OK) st = check_split(o, d, k, metric);
    if (st != KNN_OK) return st;
    if (!workspace || ((uintptr_t)workspace & 255)) return KNN_EINVAL;

    Plan p;
    st = choose_plan(nq, nr, d, k, metric, self, o, workspace_bytes, p);
    if (st != KNN_OK) return st;

    hipStream_t stream = (hipStream_t)stream_v;
    char *ws = (char *)workspace;
    float *qp = (float *)(ws + p.off_qp);
    float *rp = p.rcopy ? (float *)(ws + p.off_rp) : nullptr;
    float *cr = (float *)(ws + p.off_c);
    float *sq = (float *)(ws + p.off_sq);
    u64 *lists = (u64 *)(ws + p.off_lists);
    uint32_t *bound = (!p.fold && p.qreg && !p.tri && p.S > 1) ? (uint32_t *)(ws + p.off_bound) : nullptr;   // qreg: also the split plan

    Events ev;
    if (o.profile) {
        hipError_t e = ev.create();
        if (e != hipSuccess) {
            set_error("hipEventCreate", e);
            return KNN_EDEVICE;
        }
    }
    hipError_t e;
    ev.record(0, stream);

    // ---- prologue: norms and scaled copies ----
    const float *mu = nullptr;
    if (p.center) {
        float *m = (float *)(ws + p.off_mu);
        e = launch_col_mean(R, nr, d, p.dpad, (double *)(ws + p.off_mu + align_up((size_t)p.dpad * sizeof(float), 256)), m, stream);
        if (e != hipSuccess) { set_error("col_mean", e); return KNN_EDEVICE; }
        mu = m;
    }
    if (p.split) {
        SplitPrepArgs aq = {Q, nq, d, p.dpad, -2.f, (uint32_t *)qp, nullptr, 0, sq, bound, mu};
        e = launch_prep_split(aq, stream);
        if (e != hipSuccess) { set_error("prep_split(Q)", e); return KNN_EDEVICE; }
        SplitPrepArgs ar = {R, nr, d, p.dpad, 1.f, (uint32_t *)rp, cr, p.n_cpad, nullptr, nullptr, mu};
        e = launch_prep_split(ar, stream);
        if (e != hipSuccess) { set_error("prep_split(R)", e); return KNN_EDEVICE; }
        e = launch_reduce_max(cr, nr, (float *)(ws + p.off_sq + align_up((size_t)nq * sizeof(float), 256)), stream);
        if (e != hipSuccess) { set_error("reduce_max", e); return KNN_EDEVICE; }
        e = launch_zero_word((int32_t *)(ws + p.off_fb_words), stream);
        if (e != hipSuccess) { set_error("zero_word", e); return KNN_EDEVICE; }
        if (p.dpad != d || p.center) {
            // the second pass reads fp32 reference rows of dpad coordinates
            PrepArgs a32 = {R, nr, d, p.dpad, (int32_t)KNN_SQEUCLIDEAN, nullptr, (float *)(ws + p.off_r32), nullptr, nr, nullptr, nullptr, mu};
            e = launch_prep(a32, stream);
            if (e != hipSuccess) { set_error("prep_rows(R, fp32)", e); return KNN_EDEVICE; }
        }
    } else if (p.fold) {
        PackArgs pq = {Q, qp, nq, d, p.dpad, 64, p.matrix ? nullptr : (uint32_t *)cr};
        e = launch_pack(pq, stream);
        if (e != hipSuccess) { set_error("pack_tiles(Q)", e); return KNN_EDEVICE; }
        PackArgs pk = {R, rp, nr, d, p.dpad, KNN_FOLD_NR, nullptr};
        e = launch_pack(pk, stream);
        if (e != hipSuccess) { set_error("pack_tiles(R)", e); return KNN_EDEVICE; }
    } else if (self) {
        PrepArgs a = {R, nr, d, p.dpad, (int32_t)metric, qp, rp, cr, p.n_cpad, sq, bound, mu};
        e = launch_prep(a, stream);
        if (e != hipSuccess) { set_error("prep_rows", e); return KNN_EDEVICE; }
    } else {
        PrepArgs aq = {Q, nq, d, p.dpad, (int32_t)metric, qp, nullptr, nullptr, nq, sq, bound, mu};
        e = launch_prep(aq, stream);
        if (e != hipSuccess) { set_error("prep_rows(Q)", e); return KNN_EDEVICE; }
        PrepArgs ar = {R, nr, d, p.dpad, (int32_t)metric, nullptr, rp, cr, p.n_cpad, nullptr, nullptr, mu};
        e = launch_prep(ar, stream);
        if (e != hipSuccess) { set_error("prep_rows(R)", e); return KNN_EDEVICE; }
    }
    ev.record(1, stream);

    // ---- fused distance + selection ----
    int32_t launches = 1;
    int64_t pairs_computed = p.nq_pad * p.n_cpad;
    if (p.matrix) {
        st = run_two_phase(p, Q, nq, R, nr, d, k, metric, self_offset, qp, rp, cr, lists, ws, stream, ev,
                           launches, pairs_computed);
        if (st != KNN_OK) return st;
    } else if (p.fold) {
        FoldArgs fa;
        fa.Qpk = qp;
        fa.Rpk = rp;
        fa.lists = lists;
        fa.bound = (uint32_t *)cr;
        fa.nq = nq;
        fa.nr = nr;
        fa.nq_pad = p.nq_pad;
        fa.self_offset = self_offset;
        fa.refs_per_split = p.refs_per_split;
        fa.dpad = p.dpad;
        fa.k = k;
        fa.kcap = p.kcap;
        fa.metric = (int32_t)metric;
        fa.S = p.S;
        e = launch_fold(fa, stream);
        if (e != hipSuccess) { set_error("knn_fold", e); return KNN_EDEVICE; }
        pairs_computed = (nq + 63) / 64 * 64 * p.n_cpad;
    } else if (p.tri) {
        // one launch for the diagonal blocks, then one per round of disjoint block pairs
        float *cmax = (float *)(ws + p.off_sq + align_up((size_t)nq * sizeof(float), 256));
        e = launch_reduce_max(cr, nr, cmax, stream);
        if (e != hipSuccess) { set_error("reduce_max", e); return KNN_EDEVICE; }
        ev.record(1, stream);
        PairArgs pa;
        pa.Qp = qp;
        pa.Rp = p.rcopy ? rp : R;
        pa.cR = cr;
        pa.cmax = cmax;
        pa.lists = lists;
        pa.ldq = p.dpad;
        pa.ldr = p.rcopy ? p.dpad : d;
        pa.n = nr;
        pa.dpad = p.dpad;
        pa.k = k;
        if (p.split) pa.k = (int32_t)(nr - 1 < p.kcap ? nr - 1 : p.kcap);   // every entry of the lists live
        pa.kcap = p.kcap;
        pa.metric = (int32_t)metric;
        pa.B = p.B;
        pa.NB = p.NB;
        pa.NBp = p.NBp;
        pa.round = -1;
        e = launch_pairs_qreg(pa, p.NB, p.split, stream);
        if (e != hipSuccess) { set_error("knn_pairs_qreg(diagonal)", e); return KNN_EDEVICE; }
        for (int32_t r = 0; r + 1 < p.NBp; ++r) {
            pa.round = r;
            e = launch_pairs_qreg(pa, p.NBp / 2, p.split, stream);
            if (e != hipSuccess) { set_error("knn_pairs_qreg", e); return KNN_EDEVICE; }
        }
        launches = p.NBp;
        // padded rows actually contracted: queries in tiles of 128, references in tiles of 64
        const int64_t last = nr - (int64_t)(p.NB - 1) * p.B;
        const int64_t lq = (last + KNN_TILE - 1) / KNN_TILE * KNN_TILE, lr = (last + 63) / 64 * 64;
        const int64_t full = p.NB - 1;
        pairs_computed = full * (int64_t)p.B * p.B + lq * lr                  // diagonal blocks
                         + full * (full - 1) / 2 * (int64_t)p.B * p.B;       // pairs of full blocks
        // pairs with the ragged last block: it is the query side when it is `ba` of the circle
        // method; count the larger of the two paddings (an upper bound within 64 rows per pair)
        pairs_computed += full * (int64_t)p.B * (lq > lr ? lq : lr);
    } else {
        TileArgs t;
        t.Qp = qp;
        t.Rp = p.rcopy ? rp : R;
        t.cR = cr;
        t.lists = lists;
        t.bound = bound;
        t.ldq = p.dpad;
        t.ldr = p.rcopy ? p.dpad : d;
        t.nq = nq;
        t.nr = nr;
        t.nq_pad = p.nq_pad;
        t.self_offset = self_offset;
        t.dpad = p.dpad;
        t.k = k;
        t.kcap = p.kcap;
        t.n_qtiles = p.n_qtiles;
        t.n_rtiles = p.n_rtiles;
        t.S = p.S;
        t.rt_per_split = p.rt_per_split;
        t.nq_dev = nullptr;
        t.self_rows = nullptr;
        // the split plan keeps every entry of its lists live: as many as the lists hold, or as there are references
        const int64_t avail = nr - (self_offset >= 0 ? 1 : 0);
        if (p.split) t.k = (int32_t)(avail < p.kcap ? avail : p.kcap);
        e = p.split ? launch_tiles_split(t, p.split_waves, stream) : p.qreg ? launch_tiles_qreg(t, stream) : launch_tiles(t, stream);
        if (e != hipSuccess) {
            set_error(p.split ? "knn_tiles_split" : p.qreg ? "knn_tiles_qreg" : "knn_tiles", e);
            return KNN_EDEVICE;
        }
    }
    ev.record(2, stream);

    // ---- merge partial lists, re-score, final order ----
    FinArgs f;
    f.lists = lists;
    f.Q = Q;
    f.R = R;
    f.sq = sq;
    f.idx = idx;
    f.dist = dist;
    f.nq = nq;
    f.nq_pad = p.matrix ? nq : p.nq_pad;           // select_rows packs its lists by row count
    f.nr = nr;
    f.d = d;
    f.k = k;
    f.kcap = p.kcap;
    f.S = p.nlists;
    if (metric == KNN_L1)
        f.mode = o.rescore == 2 ? FIN_SELECT : FIN_RESCORE_L1;      // the fold's value is the distance
    else if (metric == KNN_LINF)
        f.mode = o.rescore == 2 ? FIN_SELECT : FIN_RESCORE_LINF;
    else if (metric == KNN_KL)
        f.mode = o.rescore == 2 ? FIN_ADD_SQ_SIGNED : FIN_RESCORE_KL;
    else if (metric == KNN_COSINE)
        f.mode = o.rescore == 2 ? FIN_ADD_ONE : FIN_RESCORE_COS;
    else if (metric == KNN_HELLINGER)
        f.mode = o.rescore == 2 ? FIN_ADD_SQ : FIN_RESCORE_HEL;
    else
        f.mode = o.rescore == 2 ? FIN_ADD_SQ : FIN_RESCORE_SQ;
    f.vec4 = (d % 4 == 0) ? 1 : 0;
    if (f.mode == FIN_SELECT) f.Q = nullptr;       // the fold's values are the distances: reported from the keys
    f.krs = 0;
    f.all_kept = 0;
    f.unc_rows = nullptr;
    f.unc_cap = 0;
    f.row_map = nullptr;
    f.nq_dev = nullptr;
    f.cmax = nullptr;
    f.err_a = f.err_b = 0.0;
    f.uncert = nullptr;
    if (p.split) {
        // Error of the value the split kernel selects on, p~ = fl(c_j + sum of 3 dpad bf16 products),
        // against p = |r|^2 - 2 q.r, with Q' = -2q and every fp32 value v = hi + lo + e, |e| <= 2^-16 |v|,
        // |lo| <= 2^-8 (1 + 2^-8) |v|:
        //   left out per coordinate: lo*lo + e_q R + Q' e_r     <= 3.02 * 2^-16 |Q'_c| |R_c|
        //   summed (Cauchy-Schwarz):                            <= alpha |Q'| |r|,  alpha = 3.02 * 2^-16
        //   fp32 accumulation of 3 dpad + 1 terms, any order, taken at 2^-22 per term (four times the
        //   unit roundoff of round-to-nearest, since the matrix unit's internal rounding is not
        //   specified):                                         <= beta (c_j + 1.02 |Q'| |r|)
        //   c_j = fl(|r|^2):                                    <= 2^-24 |r|^2
        // With |Q'| = 2 |q| and |r|^2 <= cmax:  E <= err_a |q| sqrt(cmax) + err_b cmax.
        const double alpha = 3.02 / 65536.0, beta = (3.0 * p.dpad + 2.0) / 4194304.0;
        f.mode = FIN_RESCORE_SQ;                   // the refinement IS the re-pricing: always on
        f.krs = (int32_t)(nr - (self_offset >= 0 ? 1 : 0) < p.kcap ? nr - (self_offset >= 0 ? 1 : 0) : p.kcap);
        f.all_kept = nr - (self_offset >= 0 ? 1 : 0) <= p.kcap ? 1 : 0;
        f.cmax = (const float *)(ws + p.off_sq + align_up((size_t)nq * sizeof(float), 256));
        f.err_a = 2.0 * (alpha + 1.02 * beta);
        f.err_b = beta + 1.0 / 8388608.0;
        // each pair once: a value may have reached its list as (p~ - c_j) + c_q, two more roundings of
        // numbers below 4 cmax
        if (p.tri) f.err_b += 1.0 / 2097152.0;
        f.uncert = (int32_t *)(ws + p.off_fb_words);
        f.unc_rows = (int32_t *)(ws + p.off_fb_rows);
        f.unc_cap = p.fb_cap;
    }
    e = launch_finalize(f, stream);
    if (e != hipSuccess) { set_error("finalize_rows", e); return KNN_EDEVICE; }
    if (p.split) {
        // Second pass: the rows the bound could not certify (up to fb_cap of them) are answered again
        // by the fp32 kernel over all references, as the fused fp32 plan would answer them.  The
        // number of such rows is only known on the device: the launches have room for fb_cap rows
        // and their workgroups beyond the count leave at once.
        int32_t *words = (int32_t *)(ws + p.off_fb_words);
        GatherArgs g;
        g.Q = Q;
        g.rows = (const int32_t *)(ws + p.off_fb_rows);
        g.count = words;
        g.q_out = (float *)(ws + p.off_fb_q);
        g.self_out = (int32_t *)(ws + p.off_fb_self);
        g.b_out = (uint32_t *)(ws + p.off_fb_bound);
        g.n_out = words + 1;
        g.left_out = o.uncertified;
        g.mu = p.center ? (const float *)(ws + p.off_mu) : nullptr;
        g.self_offset = self_offset;
        g.d = d;
        g.dpad = p.dpad;
        g.cap = p.fb_cap;
        e = launch_gather_rows(g, stream);
        if (e != hipSuccess) { set_error("gather_rows", e); return KNN_EDEVICE; }
        TileArgs t;
        t.Qp = g.q_out;
        t.Rp = (p.dpad != d || p.center) ? (const float *)(ws + p.off_r32) : R;
        t.cR = cr;
        t.lists = (u64 *)(ws + p.off_fb_lists);
        t.bound = g.b_out;
        t.ldq = p.dpad;
        t.ldr = p.dpad;
        t.nq = p.fb_cap;
        t.nr = nr;
        t.nq_pad = p.fb_cap;
        t.self_offset = -1;
        t.dpad = p.dpad;
        t.k = k;
        t.kcap = p.fb_kcap;
        t.n_qtiles = p.fb_cap / KNN_TILE;
        t.n_rtiles = p.n_rtiles;
        t.S = p.fb_S;
        t.rt_per_split = p.fb_rt_per_split;
        t.nq_dev = words + 1;
        t.self_rows = g.self_out;
        e = launch_tiles_qreg_subset(t, stream);
        if (e != hipSuccess) { set_error("knn_tiles_qreg(second pass)", e); return KNN_EDEVICE; }
        FinArgs f2 = f;
        f2.lists = t.lists;
        f2.nq = p.fb_cap;
        f2.nq_pad = p.fb_cap;
        f2.kcap = p.fb_kcap;
        f2.S = p.fb_S;
        f2.krs = 0;
        f2.uncert = nullptr;
        f2.unc_rows = nullptr;
        f2.row_map = g.rows;
        f2.nq_dev = words + 1;
        e = launch_finalize(f2, stream);
        if (e != hipSuccess) { set_error("finalize_rows(second pass)", e); return KNN_EDEVICE; }
    }
    ev.record(3, stream);

    if (o.profile) {
        e = hipEventSynchronize(ev.e[3]);
        if (e != hipSuccess) { set_error("hipEventSynchronize", e); return KNN_EDEVICE; }
        knn_profile_t *pr = o.profile;
        memset(pr, 0, sizeof(*pr));
        (void)hipEventElapsedTime(&pr->ms_prepare, ev.e[0], ev.e[1]);
        (void)hipEventElapsedTime(&pr->ms_main, ev.e[1], ev.e[2]);
        (void)hipEventElapsedTime(&pr->ms_finalize, ev.e[2], ev.e[3]);
        (void)hipEventElapsedTime(&pr->ms_total, ev.e[0], ev.e[3]);
        pr->main_launches = launches;
        pr->symmetric = (p.tri || p.msym) ? 1 : 0;
        pr->pairs_computed = pairs_computed;
        pr->two_phase = p.matrix ? (p.blocked ? 2 : 1) : 0;
        if (p.matrix && !p.blocked) (void)hipEventElapsedTime(&pr->ms_select, ev.e[4], ev.e[2]);
        if (p.matrix && p.blocked) pr->ms_select = pr->ms_main - ev.bracketed_ms();   // everything but the distance launches
    }
    return KNN_OK;
}

}  // namespace

extern "C" {

knn_status_t knn_build_ex(const float *X, int64_t n, int32_t d, int32_t k, knn_metric_t metric,
                          int32_t *idx, float *dist, void *workspace, size_t workspace_bytes,
                          void *stream, const knn_options_t *opt)
{
    if (n < 2) return KNN_EINVAL;
    return run(X, n, X, n, d, k, metric, 0, true, idx, dist, workspace, workspace_bytes, stream, opt);
}

knn_status_t knn_build(const float *X, int64_t n, int32_t d, int32_t k, knn_metric_t metric,
                       int32_t *idx, float *dist, void *workspace, size_t workspace_bytes,
                       void *stream)
{
    return knn_build_ex(X, n, d, k, metric, idx, dist, workspace, workspace_bytes, stream, nullptr);
}

knn_status_t knn_search_ex(const float *Q, int64_t nq, const float *R, int64_t nr, int32_t d,
                           int32_t k, knn_metric_t metric, int64_t self_offset, int32_t *idx,
                           float *dist, void *workspace, size_t workspace_bytes, void *stream,
                           const knn_options_t *opt)
{
    return run(Q, nq, R, nr, d, k, metric, self_offset, false, idx, dist, workspace,
               workspace_bytes, stream, opt);
}

knn_status_t knn_search(const float *Q, int64_t nq, const float *R, int64_t nr, int32_t d,
                        int32_t k, knn_metric_t metric, int64_t self_offset, int32_t *idx,
                        float *dist, void *workspace, size_t workspace_bytes, void *stream)
{
    return knn_search_ex(Q, nq, R, nr, d, k, metric, self_offset, idx, dist, workspace,
                         workspace_bytes, stream, nullptr);
}

knn_status_t knn_search_static(const float *Q, int64_t nq, const float *R, int64_t nr, int32_t d, int32_t k,
                               knn_metric_t metric, int64_t self_offset, int32_t *idx, float *dist, void *stream)
{
    g_last_error[0] = 0;
    if (!Q || !R || !idx || !dist) return KNN_EINVAL;
    // sizes first, so that a call too large for the array is refused before anything else happens
    knn_status_t st = check_sizes(nq, nr, d, k, metric, self_offset);
    if (st != KNN_OK) return st;
    knn_options_t o;
    memset(&o, 0, sizeof(o));
    Plan p;
    st = choose_plan(nq, nr, d, k, metric, false, o, KNN_STATIC_SCRATCH_BYTES, p);
    if (st != KNN_OK) return st;                     // KNN_ENOMEM: beyond what the static array holds
    hipError_t e;
    void *ws = static_scratch(&e);
    if (!ws) { set_error("hipGetSymbolAddress(scratch)", e); return KNN_EDEVICE; }
    // no profile record: run() then creates no event and allocates nothing, on host or device
    return run(Q, nq, R, nr, d, k, metric, self_offset, false, idx, dist, ws, KNN_STATIC_SCRATCH_BYTES, stream,
               nullptr);
}

size_t knn_select_workspace_bytes(int64_t m, int64_t n, int32_t k)
{
    if (m < 1 || n < 1 || k < 1 || k > n || k > KNN_MAX_K || n >= ((int64_t)1 << 31)) return 0;
    int32_t kcap, S;
    int64_t seg;
    select_plan(m, n, k, kcap, S, seg);
    return align_up((size_t)S * m * kcap * sizeof(u64), 256);
}

knn_status_t knn_select(const float *A, int64_t m, int64_t n, int64_t lda, int32_t k, int32_t *idx,
                        float *val, void *workspace, size_t workspace_bytes, void *stream_v)
{
    g_last_error[0] = 0;
    if (!A || !idx || !val) return KNN_EINVAL;
    if (m < 1 || n < 1 || lda < n || k < 1 || k > n) return KNN_EINVAL;
    if (((uintptr_t)A & 3) || ((uintptr_t)idx & 3) || ((uintptr_t)val & 3)) return KNN_EINVAL;
    if (k > KNN_MAX_K || n >= ((int64_t)1 << 31) || m >= ((int64_t)1 << 31)) return KNN_EUNSUPPORTED;
    int32_t kcap, S;
    int64_t seg;
    select_plan(m, n, k, kcap, S, seg);
    const size_t need = align_up((size_t)S * m * kcap * sizeof(u64), 256);
    if (!workspace || ((uintptr_t)workspace & 255)) return KNN_EINVAL;
    if (workspace_bytes < need) return KNN_ENOMEM;
    hipStream_t stream = (hipStream_t)stream_v;
    SelectArgs a;
    a.A = A;
    a.lists = (u64 *)workspace;
    a.m = m;
    a.n = n;
    a.lda = lda;
    a.seg = seg;
    a.k = k;
    a.kcap = kcap;
    a.S = S;
    a.vec4 = (((uintptr_t)A & 15) == 0 && lda % 4 == 0) ? 1 : 0;
    a.resume = 0;
    a.col0 = 0;
    a.M = nullptr;
    a.ldm = 0;
    a.tau_out = nullptr;
    hipError_t e = launch_select(a, stream);
    if (e != hipSuccess) { set_error("select_rows", e); return KNN_EDEVICE; }
    FinArgs f;
    memset(&f, 0, sizeof(f));
    f.lists = (const u64 *)workspace;
    f.Q = A;                                       // FIN_SELECT with a matrix: values are read back from it,
    f.nr = lda;                                    // row pitch nr
    f.idx = idx;
    f.dist = val;
    f.nq = m;
    f.nq_pad = m;
    f.k = k;
    f.kcap = kcap;
    f.S = S;
    f.mode = FIN_SELECT;
    e = launch_finalize(f, stream);
    if (e != hipSuccess) { set_error("finalize_rows(select)", e); return KNN_EDEVICE; }
    return KNN_OK;
}

size_t knn_workspace_bytes_ex(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric,
                              int32_t symmetric, const knn_options_t *opt)
{
    if (symmetric) nq = nr;
    if (symmetric && nr < 2) return 0;
    if (check_sizes(nq, nr, d, k, metric, symmetric ? 0 : -1) != KNN_OK) return 0;
    knn_options_t o;
    memset(&o, 0, sizeof(o));
    if (opt) o = *opt;
    if (check_options(o) != KNN_OK || check_split(o, d, k, metric) != KNN_OK) return 0;
    Plan p;
    make_plan(nq, nr, d, k, metric, symmetric != 0, o.r_splits, o.variant, o.symmetric, o.block_rows, o.center, p);
    return p.total;
}

size_t knn_workspace_bytes_min(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric,
                               int32_t symmetric)
{
    knn_options_t o;
    memset(&o, 0, sizeof(o));
    o.variant = KNN_PLAN_FUSED;
    return knn_workspace_bytes_ex(nq, nr, d, k, metric, symmetric, &o);
}

knn_status_t knn_plan(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric, int32_t symmetric,
                      const knn_options_t *opt, size_t workspace_bytes, knn_plan_info_t *out)
{
    if (!out) return KNN_EINVAL;
    if (symmetric) nq = nr;
    if (symmetric && nr < 2) return KNN_EINVAL;
    knn_status_t st = check_sizes(nq, nr, d, k, metric, symmetric ? 0 : -1);
    if (st != KNN_OK) return st;
    knn_options_t o;
    memset(&o, 0, sizeof(o));
    if (opt) o = *opt;
    st = check_options(o);
    if (st == KNN_OK) st = check_split(o, d, k, metric);
    if (st != KNN_OK) return st;
    Plan p;
    st = choose_plan(nq, nr, d, k, metric, symmetric != 0, o, workspace_bytes, p);
    if (st != KNN_OK) return st;
    memset(out, 0, sizeof(*out));
    out->plan = p.split ? KNN_PLAN_SPLIT_BF16 : p.matrix ? KNN_PLAN_TWO_PHASE
                : (p.qreg || p.fold)                         ? KNN_PLAN_FUSED
                                                             : KNN_PLAN_FUSED_STREAMING;
    out->symmetric = (p.tri || p.msym) ? 1 : 0;
    out->two_phase = p.matrix ? (p.blocked ? 2 : 1) : 0;
    out->main_launches = plan_launches(p, nr);
    out->workspace_bytes = p.total;
    const char *name = plan_kernel(p);
    size_t i = 0;
    for (; name[i] && i + 1 < sizeof(out->kernel); ++i) out->kernel[i] = name[i];
    out->kernel[i] = 0;
    return KNN_OK;
}

size_t knn_workspace_bytes(int64_t nq, int64_t nr, int32_t d, int32_t k, knn_metric_t metric,
                           int32_t symmetric)
{
    return knn_workspace_bytes_ex(nq, nr, d, k, metric, symmetric, nullptr);
}

knn_status_t knn_mfma_calibration(int64_t mfma_per_wave, int32_t waves_per_simd, float *sink,
                                  size_t sink_bytes, int64_t *total_waves, void *stream)
{
    g_last_error[0] = 0;
    if (mfma_per_wave < 16 || mfma_per_wave % 16 != 0 || waves_per_simd < 1 || waves_per_simd > 4 || !sink)
        return KNN_EINVAL;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) { set_error("hipDeviceGetAttribute", e); return KNN_EDEVICE; }
    const int blocks = cus * waves_per_simd;                 // 4 waves each: one per SIMD
    if (sink_bytes < (size_t)blocks * 256 * sizeof(float)) return KNN_EINVAL;
    e = launch_mfma_calibration(mfma_per_wave, blocks, sink, (hipStream_t)stream);
    if (e != hipSuccess) { set_error("mfma_only", e); return KNN_EDEVICE; }
    if (total_waves) *total_waves = (int64_t)blocks * 4;
    return KNN_OK;
}

knn_status_t knn_contraction_calibration(int32_t shape, int32_t dc, int64_t tiles_per_workgroup, const float *rows,
                                         float *sink, size_t sink_bytes, int64_t *workgroups, void *stream)
{
    g_last_error[0] = 0;
    if ((shape != 0 && shape != 1) || (dc != 16 && dc != 32 && dc != 64) || tiles_per_workgroup < 1 || !rows ||
        ((uintptr_t)rows & 15) || !sink)
        return KNN_EINVAL;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) { set_error("hipDeviceGetAttribute", e); return KNN_EDEVICE; }
    const int blocks = 2 * cus;                              // two workgroups of 4 waves per CU, as the tile kernels run
    if (sink_bytes < (size_t)blocks * 256 * sizeof(float)) return KNN_EINVAL;
    e = launch_contraction_calibration(shape, dc, tiles_per_workgroup, blocks, rows, sink, (hipStream_t)stream);
    if (e != hipSuccess) { set_error("contract_only", e); return KNN_EDEVICE; }
    if (workgroups) *workgroups = blocks;
    return KNN_OK;
}

knn_status_t knn_mfma_bf16_calibration(int64_t mfma_per_wave, int32_t waves_per_simd, int32_t chains, float *sink,
                                       size_t sink_bytes, int64_t *total_waves, void *stream)
{
    g_last_error[0] = 0;
    if (mfma_per_wave < 16 || mfma_per_wave % 16 != 0 || waves_per_simd < 1 || waves_per_simd > 4 ||
        (chains != 2 && chains != 4) || !sink)
        return KNN_EINVAL;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) { set_error("hipDeviceGetAttribute", e); return KNN_EDEVICE; }
    const int blocks = cus * waves_per_simd;                 // 4 waves each: one per SIMD
    if (sink_bytes < (size_t)blocks * 256 * sizeof(float)) return KNN_EINVAL;
    e = launch_mfma_bf16_calibration(mfma_per_wave, blocks, chains, sink, (hipStream_t)stream);
    if (e != hipSuccess) { set_error("mfma_bf16_only", e); return KNN_EDEVICE; }
    if (total_waves) *total_waves = (int64_t)blocks * 4;
    return KNN_OK;
}

knn_status_t knn_read_calibration(const float *buf, int64_t n_floats, int64_t floats_per_wave, float *sink,
                                  size_t sink_bytes, void *stream)
{
    g_last_error[0] = 0;
    if (!buf || !sink || ((uintptr_t)buf & 15) || n_floats < 2048 || n_floats % 2048 != 0 ||
        floats_per_wave < 2048 || floats_per_wave % 2048 != 0 || sink_bytes < 1024 * sizeof(float))
        return KNN_EINVAL;
    if ((n_floats + floats_per_wave - 1) / floats_per_wave > ((int64_t)1 << 32)) return KNN_EINVAL;
    hipError_t e = launch_read_calibration(buf, n_floats, floats_per_wave, sink, (hipStream_t)stream);
    if (e != hipSuccess) { set_error("read_only", e); return KNN_EDEVICE; }
    return KNN_OK;
}

knn_status_t knn_valu_calibration(int64_t pairs_per_wave, int32_t waves_per_simd, float *sink,
                                  size_t sink_bytes, int64_t *total_waves, void *stream)
{
    g_last_error[0] = 0;
    if (pairs_per_wave < 128 || pairs_per_wave % 128 != 0 || waves_per_simd < 1 || waves_per_simd > 8 || !sink)
        return KNN_EINVAL;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) { set_error("hipDeviceGetAttribute", e); return KNN_EDEVICE; }
    const int blocks = cus * waves_per_simd;
    // the kernel reads 16 operand values stored behind the part of the sink it writes
    if (sink_bytes < ((size_t)blocks * 256 + 16) * sizeof(float)) return KNN_EINVAL;
    static const float operands[16] = {0.013f, 0.171f, 0.029f, 0.257f, 0.043f, 0.311f, 0.059f, 0.127f,
                                       0.067f, 0.219f, 0.083f, 0.149f, 0.097f, 0.283f, 0.101f, 0.193f};
    e = hipMemcpyAsync(sink + (size_t)blocks * 256, operands, sizeof(operands), hipMemcpyHostToDevice,
                       (hipStream_t)stream);
    if (e != hipSuccess) { set_error("hipMemcpyAsync", e); return KNN_EDEVICE; }
    e = launch_valu_calibration(pairs_per_wave, blocks, sink, (hipStream_t)stream);
    if (e != hipSuccess) { set_error("valu_only", e); return KNN_EDEVICE; }
    if (total_waves) *total_waves = (int64_t)blocks * 4;
    return KNN_OK;
}

const char *knn_status_string(knn_status_t s)
{
    switch (s) {
    case KNN_OK: return "ok";
    case KNN_EINVAL: return "invalid argument";
    case KNN_EUNSUPPORTED: return "unsupported size";
    case KNN_ENOMEM: return "workspace too small";
    case KNN_EDEVICE: return "device error";
    }
    return "unknown status";
}

const char *knn_last_device_error(void) { return g_last_error; }

}  // extern "C"
