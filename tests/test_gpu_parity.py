"""Parity of the HIP library (through its C ABI) with the CPU oracle, on a real MI355X.

Acceptance rule (oracle/compare.py): distances within 1e-5 relative of the oracle's
double-precision value, identical neighbour sets except inside the 1e-5 band around the
k-th distance, ties to the lower index.  Where the arithmetic is exact (integer
lattice, one-hot rows, duplicated rows) the index lists must match bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import compare
from paper_0906_0231_amd import api, knn_build, knn_search, workloads

pytestmark = pytest.mark.gpu

RTOL = 1e-5


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the GPU"
    api.load_library()


def _check_rows(R, rows, self_offset, k, metric, g_idx, g_dist, strict=False, atol=0.0):
    """Oracle on the given query rows (indices into R offset by self_offset) vs GPU rows."""
    R = np.ascontiguousarray(R)
    rows = np.asarray(rows, dtype=np.int64)
    Q = R[rows + max(self_offset, 0)] if self_offset >= 0 else None
    assert Q is not None
    self_idx = rows + self_offset
    o_idx, o_dist, o_next = oracle.search(Q, R, k, metric, self_idx=self_idx)
    rep = compare.check(Q, R, metric, o_idx, o_dist, o_next, g_idx[rows], g_dist[rows],
                        self_idx=self_idx, rtol=RTOL, atol=atol, strict_ties=strict)
    _say(f"    {rep}")
    assert rep.ok, str(rep)
    return rep


def _sample_rows(n, count, seed):
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 31, 32, 63, 64, 127, 128, 129, 255, 256, n // 2 - 1, n // 2, n - 129, n - 128, n - 2, n - 1]
    # the panel walk cuts the rows into panels of 65 536: borders of the first, a middle and the last panel
    P = 65536
    mid = (n // P // 2) * P
    fixed += [P - 1, P, P + 1, mid - 1, mid, mid + P - 1, mid + P, n - P - 1, n - P, n - P + 1]
    fixed = [r for r in fixed if 0 <= r < n]
    extra = rng.choice(n, size=max(0, min(count, n) - len(fixed)), replace=False).tolist()
    return np.array(sorted(set(fixed + extra)), dtype=np.int64)


# ---------------------------------------------------------------------------
# small cases: several tiles, ragged tails in n and d, both metrics, every list capacity
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n,d,k,metric", [
    (1500, 64, 10, "sqeuclidean"),
    (777, 37, 5, "sqeuclidean"),
    (1000, 48, 20, "cosine"),
    (600, 130, 100, "sqeuclidean"),
    (515, 16, 64, "cosine"),
    (300, 1, 7, "sqeuclidean"),
    (129, 8, 128, "sqeuclidean"),
    (2, 5, 1, "sqeuclidean"),
    (70, 3, 69, "cosine"),
])
@pytest.mark.parametrize("variant", [1, 3, 4])
def test_build_small(n, d, k, metric, variant):
    _say(f"  build n={n} d={d} k={k} {metric} variant={variant}")
    X = workloads.gaussian(n, d, seed=1000 + n + d)
    res = knn_build(X.cuda(), k, metric, variant=variant)
    torch.cuda.synchronize()
    _check_rows(X.numpy(), np.arange(n), 0, k, metric, res.idx.cpu().numpy(), res.dist.cpu().numpy())


@pytest.mark.parametrize("variant", [1, 3, 4])
@pytest.mark.parametrize("splits", [1, 3, 16])
@pytest.mark.parametrize("rescore", [1, 2])
def test_split_reference_range_and_rescore(splits, rescore, variant):
    """Partial lists from several reference slices merge to the same answer; the answer
    without the re-score still meets the tolerance."""
    n, d, k = 2100, 32, 12
    _say(f"  splits={splits} rescore={rescore}")
    X = workloads.mixture(n, d, 8, seed=77)
    res = knn_build(X.cuda(), k, "sqeuclidean", r_splits=splits, rescore=rescore, variant=variant)
    torch.cuda.synchronize()
    _check_rows(X.numpy(), np.arange(n), 0, k, "sqeuclidean", res.idx.cpu().numpy(),
                res.dist.cpu().numpy())


@pytest.mark.parametrize("nq,nr,off,metric", [
    (300, 1000, -1, "sqeuclidean"),
    (257, 900, 643, "sqeuclidean"),
    (128, 128, 0, "cosine"),
    (1, 513, 512, "cosine"),
    (640, 200, -1, "sqeuclidean"),
])
@pytest.mark.parametrize("variant", [1, 3, 4])
def test_search_small(nq, nr, off, metric, variant):
    d, k = 24, 9
    _say(f"  search nq={nq} nr={nr} self_offset={off} {metric}")
    R = workloads.gaussian(nr, d, seed=5 + nr)
    if off >= 0:
        Q = R[off:off + nq].contiguous()
        self_idx = np.arange(nq) + off
    else:
        Q = workloads.gaussian(nq, d, seed=6 + nq)
        self_idx = None
    res = knn_search(Q.cuda(), R.cuda(), k, metric, self_offset=off, variant=variant)
    torch.cuda.synchronize()
    o_idx, o_dist, o_next = oracle.search(Q.numpy(), R.numpy(), k, metric, self_idx=self_idx)
    rep = compare.check(Q.numpy(), R.numpy(), metric, o_idx, o_dist, o_next,
                        res.idx.cpu().numpy(), res.dist.cpu().numpy(), self_idx=self_idx, rtol=RTOL)
    _say(f"    {rep}")
    assert rep.ok, str(rep)


# ---------------------------------------------------------------------------
# symmetric schedule (each unordered block pair evaluated once, both rows updated)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n,d,k,metric", [
    (1500, 64, 10, "sqeuclidean"),
    (777, 37, 5, "sqeuclidean"),
    (1000, 48, 20, "cosine"),
    (600, 130, 100, "sqeuclidean"),
    (515, 16, 64, "cosine"),
    (300, 1, 7, "sqeuclidean"),
    (129, 8, 128, "sqeuclidean"),
    (2, 5, 1, "sqeuclidean"),
    (2100, 256, 12, "sqeuclidean"),
    (4096, 64, 10, "sqeuclidean"),
])
def test_build_symmetric(n, d, k, metric):
    _say(f"  symmetric build n={n} d={d} k={k} {metric}")
    X = workloads.gaussian(n, d, seed=2000 + n + d)
    res = knn_build(X.cuda(), k, metric, symmetric=1, profile=True)
    torch.cuda.synchronize()
    assert res.profile.symmetric == 1 and res.profile.main_launches >= 2
    _check_rows(X.numpy(), np.arange(n), 0, k, metric, res.idx.cpu().numpy(), res.dist.cpu().numpy())


def test_symmetric_equals_full_square():
    """Both schedules select from the same fp32 products; on data without near-ties the
    answers are identical."""
    X = workloads.mixture(5000, 96, 12, seed=31).cuda()
    a = knn_build(X, 15, symmetric=1)
    b = knn_build(X, 15, symmetric=2)
    torch.cuda.synchronize()
    assert torch.equal(a.idx, b.idx) and torch.equal(a.dist, b.dist)
    c = knn_build(X, 15, symmetric=1)
    torch.cuda.synchronize()
    assert torch.equal(a.idx, c.idx) and torch.equal(a.dist, c.dist)     # and deterministic


@pytest.mark.parametrize("n,d,k,sym,launches", [
    (131072, 64, 10, 1, 1024),   # fused, blocks of 128 rows: 512 pairs per round, 1023 rounds + the diagonal
    (150000, 64, 10, 0, 1),      # 586 blocks of 256 rows leave the rounds 57 % full: the fused square is cheaper
    (262144, 64, 10, 1, 1024),   # fused, blocks of 256 rows
    (262144, 64, 100, 0, 1),     # long lists: the mirror merges make the triangle no cheaper yet (and at d = 64 stores would bound the two-phase form)
    (150000, 128, 100, 1, 15),   # beyond 72 GiB of matrix: two-phase by pairs of row panels (3 panels: 6 blocks, 9 selections)
    (300000, 128, 10, 1, 40),    # the same for short lists (5 panels: 15 blocks, 25 selections)
    (20000, 256, 100, 1, 2),     # the shape of the paper's Table 1: matrix written out, each pair once
    (40000, 64, 10, 1, 2),       # small enough for the two-phase form whatever d and k
    (60000, 64, 10, 0, 1),       # d = 64 and not small: the matrix would cost more than it saves
    (60000, 128, 10, 1, 2),      # d = 128: it pays
])
def test_default_schedule_choice(n, d, k, sym, launches):
    """With no option set the library takes the two-phase form where the matrix is cheap next
    to the arithmetic it saves, else the symmetric schedule where its rounds fill the device,
    else the fused square.  Sampled rows are checked against the oracle either way."""
    _say(f"  default schedule n={n} d={d} k={k}")
    X = workloads.mixture(n, d, 32, seed=77)
    res = knn_build(X.cuda(), k, profile=True)
    torch.cuda.synchronize()
    assert res.profile.symmetric == sym
    assert res.profile.main_launches == launches
    rows = _sample_rows(n, 64, seed=n % 97)
    _check_rows(X.numpy(), rows, 0, k, "sqeuclidean", res.idx.cpu().numpy(), res.dist.cpu().numpy())


# ---------------------------------------------------------------------------
# two-phase form walked block by block (pairs of row panels, lists continued from block to block)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n,d,k,metric,panel", [
    (1500, 40, 10, "sqeuclidean", 256),      # 6 panels, ragged last one (220 rows)
    (1500, 40, 10, "sqeuclidean", 1024),     # 2 panels
    (2049, 64, 100, "hellinger", 512),       # long lists; last panel of a single row
    (777, 37, 5, "cosine", 256),
    (1300, 24, 33, "l1", 256),               # the fold kernel, same walk
    (1300, 24, 12, "linf", 512),
    (600, 130, 128, "l1", 256),
    (5000, 256, 16, "sqeuclidean", 2048),
    (1500, 300, 10, "cosine", 512),          # d > 256: the streaming distance kernel, same walk
    (1100, 1030, 100, "sqeuclidean", 256),
])
def test_two_phase_by_panel_pairs(n, d, k, metric, panel):
    _say(f"  two-phase by panel pairs n={n} d={d} k={k} {metric} panel={panel}")
    gen = workloads.uniform_rows if metric == "hellinger" else workloads.gaussian
    X = gen(n, d, seed=9000 + n + d)
    res = knn_build(X.cuda(), k, metric, variant=4, block_rows=panel, profile=True)
    torch.cuda.synchronize()
    assert res.profile.two_phase == 2 and res.profile.symmetric == 1
    G = -(-n // ((panel + 255) // 256 * 256))
    assert res.profile.main_launches == G * (G + 1) // 2 + G * G      # one block per pair, one selection per block and side
    _check_rows(X.numpy(), np.arange(n), 0, k, metric, res.idx.cpu().numpy(), res.dist.cpu().numpy())
    whole = knn_build(X.cuda(), k, metric, variant=4, profile=True)
    torch.cuda.synchronize()
    assert whole.profile.two_phase == 1
    assert torch.equal(whole.idx, res.idx) and torch.equal(whole.dist, res.dist)


def test_symmetric_exact_ties():
    n, k = 2000, 6
    X = torch.arange(n, dtype=torch.float32)[:, None].contiguous()
    res = knn_build(X.cuda(), k, symmetric=1)
    torch.cuda.synchronize()
    _check_rows(X.numpy(), np.arange(n), 0, k, "sqeuclidean", res.idx.cpu().numpy(),
                res.dist.cpu().numpy(), strict=True)
    E = torch.eye(200, dtype=torch.float32)
    for metric in ("sqeuclidean", "cosine"):
        res = knn_build(E.cuda(), 17, metric, symmetric=1)
        torch.cuda.synchronize()
        _check_rows(E.numpy(), np.arange(200), 0, 17, metric, res.idx.cpu().numpy(),
                    res.dist.cpu().numpy(), strict=True)
    base = workloads.gaussian(300, 20, seed=9)
    D = base.repeat_interleave(2, dim=0).contiguous()
    res = knn_build(D.cuda(), 4, symmetric=1)
    torch.cuda.synchronize()
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    assert np.array_equal(gi[:, 0], np.arange(600) ^ 1) and np.all(gd[:, 0] == 0.0)
    _check_rows(D.numpy(), np.arange(600), 0, 4, "sqeuclidean", gi, gd, atol=1e-30)


# ---------------------------------------------------------------------------
# Hellinger distance, the distance of the paper's experiment (Sect. 7)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n,d,k,sym", [(1200, 64, 10, 2), (900, 50, 100, 2), (1500, 256, 20, 1)])
def test_hellinger(n, d, k, sym):
    X = workloads.uniform_rows(n, d, seed=60 + n)
    res = knn_build(X.cuda(), k, "hellinger", symmetric=sym)
    torch.cuda.synchronize()
    _check_rows(X.numpy(), np.arange(n), 0, k, "hellinger", res.idx.cpu().numpy(), res.dist.cpu().numpy())


def test_hellinger_perfect_squares_exact():
    """Inputs a^2 with small integer a: every distance is an integer, ties go to the lower index."""
    rng = np.random.default_rng(12)
    A = rng.integers(0, 12, size=(700, 6)).astype(np.float32)
    X = torch.from_numpy(A * A)
    res = knn_build(X.cuda(), 9, "hellinger")
    torch.cuda.synchronize()
    _check_rows(X.numpy(), np.arange(700), 0, 9, "hellinger", res.idx.cpu().numpy(),
                res.dist.cpu().numpy(), strict=True)


def test_hellinger_sparse_histograms():
    """Rows that are mostly exact zeros, with a few denormal entries: the square roots of the
    re-pricing take their exact (zero) and their slow (denormal) branch."""
    rng = np.random.default_rng(77)
    n, d = 1300, 96
    A = rng.random((n, d)).astype(np.float32)
    A[rng.random((n, d)) < 0.7] = 0.0
    A[rng.random((n, d)) < 0.02] = np.float32(3e-40)
    A[:, 0] += 0.01                               # no empty row
    X = torch.from_numpy((A / A.sum(axis=1, keepdims=True)).astype(np.float32))
    for variant in (3, 4):
        res = knn_build(X.cuda(), 12, "hellinger", variant=variant)
        torch.cuda.synchronize()
        _check_rows(X.numpy(), np.arange(n), 0, 12, "hellinger", res.idx.cpu().numpy(), res.dist.cpu().numpy())


def test_paper_experiment_shape():
    """n = 10 000, d = 256, k = 100, Hellinger: the smallest column of the paper's Table 1."""
    w = workloads.config(6, n=10000)
    res = knn_build(w.R.cuda(), w.k, w.metric, profile=True)
    torch.cuda.synchronize()
    _say(f"    gpu: {res.profile.ms_total:.1f} ms total")
    rows = _sample_rows(w.n, 512, seed=6)
    _check_rows(w.R.numpy(), rows, 0, w.k, w.metric, res.idx.cpu().numpy(), res.dist.cpu().numpy())


def test_search_equals_build():
    """knn_build(X) == knn_search(X, X, self_offset=0), bit for bit."""
    X = workloads.gaussian(900, 40, seed=3).cuda()
    a = knn_build(X, 11)
    b = knn_search(X, X, 11, self_offset=0)
    torch.cuda.synchronize()
    assert torch.equal(a.idx, b.idx) and torch.equal(a.dist, b.dist)


# ---------------------------------------------------------------------------
# exact cases: ties must go to the lower index, bit-exact distances
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("variant", [1, 3, 4])
def test_lattice_exact(variant):
    n, k = 2000, 6
    X = torch.arange(n, dtype=torch.float32)[:, None].contiguous()
    res = knn_build(X.cuda(), k, variant=variant)
    torch.cuda.synchronize()
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    _check_rows(X.numpy(), np.arange(n), 0, k, "sqeuclidean", gi, gd, strict=True)
    assert gi[1000].tolist() == [999, 1001, 998, 1002, 997, 1003]
    assert gd[1000].tolist() == [1, 1, 4, 4, 9, 9]


@pytest.mark.parametrize("kw", [
    dict(variant=4, block_rows=512),                        # two-phase by pairs of row panels
    dict(symmetric=1, block_rows=128),                      # fused tournament of block pairs
])
def test_ties_across_panels(kw):
    """Ties across block boundaries: a lattice on a line (every distance tied between the two
    sides) and a set where every pair is equidistant (the k lowest indices must win, whichever
    panel or round brings them)."""
    n, k = 2000, 6
    X = torch.arange(n, dtype=torch.float32)[:, None].contiguous()
    res = knn_build(X.cuda(), k, **kw)
    torch.cuda.synchronize()
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    _check_rows(X.numpy(), np.arange(n), 0, k, "sqeuclidean", gi, gd, strict=True)
    assert gi[1024].tolist() == [1023, 1025, 1022, 1026, 1021, 1027]
    n, k = 1500, 17
    E = torch.eye(n, dtype=torch.float32)
    res = knn_build(E.cuda(), k, **kw)
    torch.cuda.synchronize()
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    for i in (0, 1, 16, 17, 18, 511, 512, 1023, 1024, 1499):
        assert gi[i].tolist() == [j for j in range(n) if j != i][:k]
    assert np.all(gd == 2.0)


@pytest.mark.parametrize("n,d,k,panel", [(1536, 48, 8, 512), (2300, 256, 20, 768), (3000, 33, 3, 256),
                                         (1400, 300, 6, 512), (1200, 520, 40, 256)])   # d > 256: the streaming kernel filters alike
def test_panel_pairs_when_the_neighbours_come_late(n, d, k, panel):
    """Walked by panel pairs, blocks that cannot change a row's list are not stored (a row's
    threshold after the panels it has seen filters what later blocks write).  Here the true
    neighbours of the first rows sit in the last panel and those of the last rows in the first,
    and the middle is far from both: the thresholds stay loose until the very last blocks."""
    _say(f"  neighbours in the last panel n={n} d={d} k={k} panel={panel}")
    third = n // 3
    A = workloads.gaussian(third, d, seed=31 + n)
    far = workloads.gaussian(n - 2 * third, d, seed=32 + n) * 3.0 + 4.0
    near = A + 0.05 * workloads.gaussian(third, d, seed=33 + n)
    X = torch.cat([A, far, near]).contiguous()
    res = knn_build(X.cuda(), k, variant=4, block_rows=panel, profile=True)
    torch.cuda.synchronize()
    assert res.profile.two_phase == 2
    _check_rows(X.numpy(), np.arange(n), 0, k, "sqeuclidean", res.idx.cpu().numpy(), res.dist.cpu().numpy())
    assert (res.idx[:third, 0].cpu() == torch.arange(third) + (n - third)).all()


def test_ties_across_panels_streaming_kernel():
    """d > 256, walked by panel pairs with thresholds: a lattice on a line embedded in 300
    coordinates (every distance exact, every k-th distance tied between the two sides, values AT
    the thresholds that filter the stores) and a set where every pair is equidistant."""
    n, k = 1500, 6
    X = torch.zeros((n, 300), dtype=torch.float32)
    X[:, 17] = torch.arange(n, dtype=torch.float32)
    res = knn_build(X.cuda(), k, variant=4, block_rows=512, profile=True)
    torch.cuda.synchronize()
    assert res.profile.two_phase == 2
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    _check_rows(X.numpy(), np.arange(n), 0, k, "sqeuclidean", gi, gd, strict=True)
    assert gi[1024].tolist() == [1023, 1025, 1022, 1026, 1021, 1027]
    E = torch.zeros((600, 600), dtype=torch.float32)
    E[torch.arange(600), torch.arange(600)] = 1.0
    res = knn_build(E.cuda(), 17, variant=4, block_rows=256)
    torch.cuda.synchronize()
    gi = res.idx.cpu().numpy()
    for i in (0, 1, 255, 256, 257, 511, 512, 599):
        assert gi[i].tolist() == [j for j in range(600) if j != i][:17]
    _check_rows(E.numpy(), np.arange(600), 0, 17, "sqeuclidean", gi, res.dist.cpu().numpy(), strict=True)


@pytest.mark.parametrize("variant", [1, 3, 4])
@pytest.mark.parametrize("metric", ["sqeuclidean", "cosine"])
def test_all_equidistant(metric, variant):
    n, k = 200, 17
    X = torch.eye(n, dtype=torch.float32)
    res = knn_build(X.cuda(), k, metric, variant=variant)
    torch.cuda.synchronize()
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    for i in (0, 1, 16, 17, 18, 127, 128, 199):
        assert gi[i].tolist() == [j for j in range(n) if j != i][:k]
    assert np.all(gd == (2.0 if metric == "sqeuclidean" else 1.0))
    _check_rows(X.numpy(), np.arange(n), 0, k, metric, gi, gd, strict=True)


@pytest.mark.parametrize("variant", [1, 3, 4])
def test_duplicate_rows(variant):
    base = workloads.gaussian(300, 20, seed=9)
    X = base.repeat_interleave(2, dim=0).contiguous()
    res = knn_build(X.cuda(), 4, variant=variant)
    torch.cuda.synchronize()
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    assert np.array_equal(gi[:, 0], np.arange(600) ^ 1)
    assert np.all(gd[:, 0] == 0.0)              # the re-score makes the twin's distance exactly 0
    # each row's 2nd/3rd neighbours are another duplicated pair: an exact tie, lower index first
    assert np.all(gi[:, 1] + 1 == gi[:, 2]) and np.all(gi[:, 1] % 2 == 0)
    _check_rows(X.numpy(), np.arange(600), 0, 4, "sqeuclidean", gi, gd, atol=1e-30)


@pytest.mark.parametrize("variant", [1, 3, 4])
def test_deterministic(variant):
    X = workloads.mixture(3000, 64, 16, seed=4).cuda()
    a = knn_build(X, 10, variant=variant)
    b = knn_build(X, 10, variant=variant)
    torch.cuda.synchronize()
    assert torch.equal(a.idx, b.idx) and torch.equal(a.dist, b.dist)


def test_nondefault_stream_and_caller_buffers():
    X = workloads.gaussian(1000, 32, seed=8)
    Xd = X.cuda()
    idx = torch.empty((1000, 5), dtype=torch.int32, device="cuda")
    dist = torch.empty((1000, 5), dtype=torch.float32, device="cuda")
    ws = torch.empty(api.knn_workspace_bytes(1000, 1000, 32, 5, symmetric=True), dtype=torch.uint8,
                     device="cuda")
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        knn_build(Xd, 5, workspace=ws, out=(idx, dist))
    s.synchronize()
    _check_rows(X.numpy(), np.arange(1000), 0, 5, "sqeuclidean", idx.cpu().numpy(), dist.cpu().numpy())


def test_mfma_calibration_runs():
    """The matrix-instruction-only kernel: right amount of work, a plausible rate, and the
    sink-size check."""
    from paper_0906_0231_amd import knn_mfma_calibration
    tf, ms = knn_mfma_calibration(1 << 14, 2)
    assert ms > 0 and 1.0 < tf < 200.0
    lib = api.load_library()
    sink = torch.empty(64, dtype=torch.float32, device="cuda")
    st = lib.knn_mfma_calibration(1024, 2, sink.data_ptr(), sink.numel() * 4, None, None)
    assert st == api.KNN_EINVAL
    from paper_0906_0231_amd import knn_mfma_bf16_calibration
    for chains in (4, 2):
        tf, ms = knn_mfma_bf16_calibration(1 << 14, 2, chains)
        assert ms > 0 and 10.0 < tf < 3000.0
    from paper_0906_0231_amd import knn_contraction_calibration
    for shape in (0, 1):
        for dc in (16, 32, 64):
            tf, ms = knn_contraction_calibration(shape, dc, 64)
            assert ms > 0 and 1.0 < tf < 200.0
    from paper_0906_0231_amd import knn_valu_calibration
    tops, ms = knn_valu_calibration(1 << 14, 2)
    assert ms > 0 and 1.0 < tops < 100.0
    st = lib.knn_valu_calibration(1024, 2, sink.data_ptr(), sink.numel() * 4, None, None)
    assert st == api.KNN_EINVAL
    from paper_0906_0231_amd import knn_read_calibration
    buf = torch.full((1 << 24,), 3.0, dtype=torch.float32, device="cuda")
    buf[12345678] = -7.0
    gbs, ms = knn_read_calibration(buf, 1 << 16)
    assert ms > 0 and 10.0 < gbs < 20000.0


def test_device_error_paths():
    X = workloads.gaussian(100, 8, seed=1).cuda()
    with pytest.raises(api.KnnError) as e:
        knn_build(X, 100)
    assert e.value.status == api.KNN_EINVAL
    with pytest.raises(api.KnnError) as e:
        knn_build(X, 5, workspace=torch.empty(512, dtype=torch.uint8, device="cuda"))
    assert e.value.status == api.KNN_ENOMEM


# ---------------------------------------------------------------------------
# the benchmark configurations at full size (oracle on sampled rows where the full
# oracle would take hours)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("variant", [1, 3, 4])
def test_config1_full(variant):
    w = workloads.config(1)
    _say(f"  {w.name} variant={variant}")
    res = knn_build(w.R.cuda(), w.k, w.metric, variant=variant)
    torch.cuda.synchronize()
    _check_rows(w.R.numpy(), np.arange(w.n), 0, w.k, w.metric, res.idx.cpu().numpy(),
                res.dist.cpu().numpy())


def _full_size(which, sample, variant=0, two_phase=None, symmetric=0, kernel=None):
    w = workloads.config(which)
    _say(f"  {w.name}: generated (variant {variant}, symmetric {symmetric})")
    Rd = w.R.cuda()
    if w.symmetric:
        res = knn_build(Rd, w.k, w.metric, variant=variant, symmetric=symmetric, profile=True)
    else:
        res = knn_search(Rd[:w.nq], Rd, w.k, w.metric, self_offset=0, variant=variant, profile=True)
    torch.cuda.synchronize()
    if two_phase is not None:
        assert res.profile.two_phase == two_phase and res.plan.two_phase == two_phase
    if kernel is not None:
        assert res.plan.kernel.decode() == kernel
    _say(f"    gpu: {res.profile.ms_total:.1f} ms total, {res.profile.ms_main:.1f} ms main stage, {res.plan}")
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    del Rd
    rows = _sample_rows(w.nq, sample, seed=which)
    _check_rows(w.R.numpy(), rows, 0, w.k, w.metric, gi, gd)
    # properties that hold at any size, on every row
    assert np.all(np.diff(gd, axis=1) >= 0)
    assert not np.any(gi == np.arange(w.nq, dtype=np.int64)[:, None])
    assert gi.min() >= 0 and gi.max() < w.n
    s = np.sort(gi, axis=1)
    assert np.all(s[:, 1:] != s[:, :-1])


# Oracle samples at full size: 1024 query rows for configs 2-4 and the Table-1 shape, 256 for
# config 5 (8.4 million references each), always with rows at tile borders and at the borders of
# the first, a middle and the last row panel.
@pytest.mark.parametrize("variant,two_phase", [(0, 1), (3, 0)])
def test_config2_full(variant, two_phase):
    _full_size(2, 1024, variant, two_phase)      # by default the two-phase form (d = 128, matrix of 16 GiB)


@pytest.mark.parametrize("symmetric,two_phase,kernel", [(0, 2, "knn_dist_qreg"), (1, 0, "knn_pairs_qreg")])
def test_config3_full(symmetric, two_phase, kernel):
    """The headline workload in the plan bench.py times (by pairs of row panels, stores filtered
    by the lists' thresholds) and in the fused symmetric schedule."""
    _full_size(3, 1024, two_phase=two_phase, symmetric=symmetric, kernel=kernel)


@pytest.mark.parametrize("variant,two_phase,kernel", [(0, 2, "knn_dist_stream"), (3, 0, "knn_tiles")])
def test_config4_full(variant, two_phase, kernel):
    """d = 1024: by default the streaming distance kernel by pairs of row panels; on request the
    fused streaming kernel (the register-resident one stops at d = 256)."""
    _full_size(4, 1024, variant, two_phase, symmetric=2 if variant == 3 else 0, kernel=kernel)


def test_config5_full():
    _full_size(5, 256, kernel="knn_tiles_qreg")


def test_search_full_size_with_self_offset():
    """A query block from the middle of a large reference set: queries = rows [2^19, 2^19 + 65 536)
    of a 2^20 x 128 mixture, each excluding itself by its offset row number."""
    nr, nq, d, k, off = 1 << 20, 65536, 128, 16, 1 << 19
    R = workloads.mixture(nr, d, 256, seed=workloads.BASE_SEED + 55)
    Rd = R.cuda()
    res = knn_search(Rd[off:off + nq], Rd, k, "sqeuclidean", self_offset=off, profile=True)
    torch.cuda.synchronize()
    _say(f"    gpu: {res.profile.ms_total:.1f} ms total, {res.plan}")
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    del Rd
    assert not np.any(gi == (np.arange(nq, dtype=np.int64) + off)[:, None])
    rng = np.random.default_rng(55)
    rows = np.unique(np.concatenate([rng.choice(nq, 500, replace=False), [0, 127, 128, nq // 2, nq - 1]]))
    Rh = R.numpy()
    o_idx, o_dist, o_next = oracle.search(Rh[rows + off], Rh, k, "sqeuclidean", self_idx=rows + off)
    rep = compare.check(Rh[rows + off], Rh, "sqeuclidean", o_idx, o_dist, o_next, gi[rows], gd[rows],
                        self_idx=rows + off, rtol=RTOL)
    _say(f"    {rep}")
    assert rep.ok, str(rep)


@pytest.mark.parametrize("variant,two_phase", [(0, 1), (3, 0)])
def test_paper_table1_shape_full(variant, two_phase):
    """n = 80 000, d = 256, k = 100, Hellinger (the largest row of the paper's Table 1): the
    two-phase form by default, the fused kernel on request."""
    _full_size(6, 1024, variant, two_phase)


# ---------------------------------------------------------------------------
# the plan follows the workspace; both sides of every rule of the default choice
# ---------------------------------------------------------------------------
def test_plan_follows_the_workspace():
    """With default options the library takes the preferred plan when the workspace holds it and
    the fused plan when it does not -- no error -- and says which; both answers meet the rule."""
    n, d, k = 20000, 128, 10
    X = workloads.mixture(n, d, 16, seed=4242)
    Xd = X.cuda()
    big = api.knn_workspace_bytes(n, n, d, k, symmetric=True)
    small = api.knn_workspace_bytes_min(n, n, d, k, symmetric=True)
    assert small < big // 8
    rows = _sample_rows(n, 200, seed=5)
    for nbytes, two_phase, kernel in ((big, 1, "knn_dist_qreg"), (small, 0, "knn_tiles_qreg"), (big - 256, 0, "knn_tiles_qreg")):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        res = knn_build(Xd, k, workspace=ws, profile=True)
        torch.cuda.synchronize()
        assert res.plan.two_phase == two_phase == res.profile.two_phase
        assert res.plan.kernel.decode() == kernel and res.plan.workspace_bytes <= nbytes
        _check_rows(X.numpy(), rows, 0, k, "sqeuclidean", res.idx.cpu().numpy(), res.dist.cpu().numpy())
        del ws
    with pytest.raises(api.KnnError) as e:
        knn_build(Xd, k, workspace=torch.empty(small - 256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == api.KNN_ENOMEM
    with pytest.raises(api.KnnError) as e:          # a plan asked for by name is not replaced
        knn_build(Xd, k, variant=4, workspace=torch.empty(small, dtype=torch.uint8, device="cuda"))
    assert e.value.status == api.KNN_ENOMEM


@pytest.mark.parametrize("n,d,k,two_phase,sym", [
    (30000, 64, 32, 1, 1),        # k = 32 / 33: lists of 32 / 64 entries; long lists always take the two-phase form
    (60000, 64, 32, 0, 0),
    (60000, 64, 33, 1, 1),
    (60000, 96, 10, 0, 0),        # d = 96 / 97 (padded to 96 / 128): from 128 on computing each pair once pays
    (60000, 97, 10, 1, 1),
    (49152, 64, 10, 1, 1),        # d = 64: two-phase up to 49 152 rows
    (49152 + 128, 64, 10, 0, 0),
    (138880, 128, 10, 1, 1),      # the matrix whole up to 72 GiB ...
    (139008, 128, 10, 2, 1),      # ... one tile more: by pairs of row panels
])
def test_both_sides_of_the_plan_rules(n, d, k, two_phase, sym):
    """One case on each side of every threshold of the default plan choice, each checked against
    the oracle on sampled rows (not only for the plan it takes)."""
    _say(f"  plan rule n={n} d={d} k={k}")
    X = workloads.mixture(n, d, 32, seed=n % 1000 + d)
    res = knn_build(X.cuda(), k)
    torch.cuda.synchronize()
    _say(f"    {res.plan}")
    assert res.plan.two_phase == two_phase and res.plan.symmetric == sym
    rows = _sample_rows(n, 96, seed=n % 89)
    _check_rows(X.numpy(), rows, 0, k, "sqeuclidean", res.idx.cpu().numpy(), res.dist.cpu().numpy())


@pytest.mark.parametrize("nr,two_phase", [(130944, 1), (131072, 0)])
def test_search_plan_rule_at_4_gib(nr, two_phase):
    """Queries against a separate reference set: the matrix is written out while it is at most
    4 GiB (8192 x (130944 + 64) x 4 bytes is just below, 8192 x (131072 + 64) x 4 just above)."""
    nq, d, k = 8192, 64, 16
    R = workloads.mixture(nr, d, 32, seed=nr % 1000)
    Q = workloads.mixture(nq, d, 32, seed=7)
    res = knn_search(Q.cuda(), R.cuda(), k)
    torch.cuda.synchronize()
    _say(f"    {res.plan}")
    assert res.plan.two_phase == two_phase
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([rng.choice(nq, 96, replace=False), [0, nq - 1]]))
    o_idx, o_dist, o_next = oracle.search(Q.numpy()[rows], R.numpy(), k, "sqeuclidean")
    rep = compare.check(Q.numpy()[rows], R.numpy(), "sqeuclidean", o_idx, o_dist, o_next,
                        res.idx.cpu().numpy()[rows], res.dist.cpu().numpy()[rows], rtol=RTOL)
    _say(f"    {rep}")
    assert rep.ok, str(rep)
