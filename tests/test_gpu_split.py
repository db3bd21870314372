"""The split-precision experiment (KNN_PLAN_SPLIT_BF16): operands cut into two bf16 pieces, three
bf16 matrix products per pair, used as a filter whose survivors are priced exactly.  Its answers
are held to the same rule against the CPU oracle as every other plan's; where the arithmetic is
exact (small integers survive the split) the index lists must match bit for bit.  The number of
rows left unproven (neither certified by the error bound nor taken by the fp32 second pass) is
printed; it does not enter the verdict -- the comparison with the oracle does."""
import numpy as np
import pytest
import torch

import oracle
from oracle import compare
from paper_0906_0231_amd import api, knn_build, knn_search, workloads

pytestmark = pytest.mark.gpu
RTOL = 1e-5
SPLIT = api.PLAN_SPLIT_BF16


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the GPU"
    api.load_library()


def _check(Q, R, self_idx, k, g_idx, g_dist, strict=False, atol=0.0):
    o_idx, o_dist, o_next = oracle.search(Q, R, k, "sqeuclidean", self_idx=self_idx)
    rep = compare.check(Q, R, "sqeuclidean", o_idx, o_dist, o_next, g_idx, g_dist, self_idx=self_idx,
                        rtol=RTOL, atol=atol, strict_ties=strict)
    _say(f"    {rep}")
    assert rep.ok, str(rep)
    return rep


def _build(X, k, **kw):
    unc = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    res = knn_build(X.cuda(), k, variant=SPLIT, uncertified=unc, **kw)
    torch.cuda.synchronize()
    assert res.plan.plan == SPLIT
    assert res.plan.kernel == (b"knn_pairs_qreg" if res.plan.symmetric else b"knn_tiles_split")
    n_unc = int(unc.item())
    assert 0 <= n_unc <= X.shape[0]
    return res, n_unc


# several query tiles of 256 and reference tiles of 64, ragged tails in n and d, every list
# capacity (the lists hold k plus a margin: 16 for k <= 14, 128 for k = 100), k = n - 1, slices
@pytest.mark.parametrize("n,d,k,splits", [
    (1500, 64, 10, 0),
    (777, 37, 5, 0),
    (600, 130, 100, 3),
    (515, 16, 60, 1),
    (300, 1, 7, 0),
    (129, 8, 112, 0),
    (2, 5, 1, 0),
    (70, 3, 69, 0),
    (2100, 256, 12, 7),
    (4100, 200, 14, 0),
])
@pytest.mark.parametrize("symmetric", [2, 1])
def test_split_build_small(n, d, k, splits, symmetric):
    _say(f"  split build n={n} d={d} k={k} splits={splits} symmetric={symmetric}")
    X = workloads.gaussian(n, d, seed=7000 + n + d)
    res, n_unc = _build(X, k, r_splits=splits, symmetric=symmetric)
    assert res.plan.symmetric == (1 if symmetric == 1 else 0)
    _say(f"    rows left unproven: {n_unc} of {n}")
    _check(X.numpy(), X.numpy(), np.arange(n), k, res.idx.cpu().numpy(), res.dist.cpu().numpy())


@pytest.mark.parametrize("nq,nr,off", [(300, 1000, -1), (257, 900, 643), (128, 128, 0), (1, 513, 512), (640, 200, -1)])
def test_split_search_small(nq, nr, off):
    d, k = 24, 9
    _say(f"  split search nq={nq} nr={nr} self_offset={off}")
    R = workloads.gaussian(nr, d, seed=5 + nr)
    Q = R[off:off + nq].contiguous() if off >= 0 else workloads.gaussian(nq, d, seed=6 + nq)
    self_idx = np.arange(nq) + off if off >= 0 else None
    res = knn_search(Q.cuda(), R.cuda(), k, self_offset=off, variant=SPLIT)
    torch.cuda.synchronize()
    _check(Q.numpy(), R.numpy(), self_idx, k, res.idx.cpu().numpy(), res.dist.cpu().numpy())


@pytest.mark.parametrize("symmetric", [2, 1])
def test_split_exact_ties(symmetric):
    """Small integers are exact in two bf16 pieces (16 bits), their products and sums exact in
    fp32: a lattice on a line, one-hot rows (every pair equidistant) and duplicated rows must give
    the oracle's index lists bit for bit, ties to the lower index -- in the full square and with
    each pair evaluated once (blocks of 128 rows: ties across block borders and rounds)."""
    n, k = 2000, 6
    def build(X, k):
        return _build(X, k, symmetric=symmetric, block_rows=128 if symmetric == 1 else 0)
    X = torch.arange(n, dtype=torch.float32)[:, None].contiguous()
    res, n_unc = build(X, k)
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    _check(X.numpy(), X.numpy(), np.arange(n), k, gi, gd, strict=True)
    assert gi[1000].tolist() == [999, 1001, 998, 1002, 997, 1003] and gd[1000].tolist() == [1, 1, 4, 4, 9, 9]
    E = torch.eye(256, dtype=torch.float32)
    res, n_unc = build(E, 17)
    _say(f"    one-hot rows left unproven: {n_unc} of 256 (every pair ties: all 256 go through the second pass)")
    assert n_unc == 0
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    for i in (0, 1, 16, 17, 18, 127, 128, 255):
        assert gi[i].tolist() == [j for j in range(256) if j != i][:17]
    assert np.all(gd == 2.0)
    base = workloads.gaussian(300, 20, seed=9)
    D = base.repeat_interleave(2, dim=0).contiguous()
    res, n_unc = build(D, 4)
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    assert np.array_equal(gi[:, 0], np.arange(600) ^ 1) and np.all(gd[:, 0] == 0.0)
    _check(D.numpy(), D.numpy(), np.arange(600), 4, gi, gd, atol=1e-30)


def test_split_second_pass_and_its_overflow():
    """Totally tied data (50 distinct small-integer points, each repeated n/50 times: every row has
    more than K' references at distance 0, all values exact in every plan): the bound can certify
    nothing, so the fp32 second pass answers up to 4096 rows and the rest keep the filter's answer
    -- all of them the oracle's lists bit for bit.  With 3000 rows everything fits the second pass,
    with 6000 rows 1904 are left over and counted."""
    rng = np.random.default_rng(21)
    base = rng.integers(0, 3, size=(50, 8)).astype(np.float32)
    for n, left_some, symmetric in ((3000, False, 2), (6000, True, 2), (3000, False, 1)):
        X = torch.from_numpy(base[np.arange(n) % 50].copy())
        res, left = _build(X, 9, symmetric=symmetric)
        _say(f"    n={n}: rows left unproven after the second pass: {left}")
        assert left == (n - 4096 if left_some else 0)
        o_idx, o_dist, _ = oracle.build_knn(X.numpy(), 9)
        assert np.array_equal(res.idx.cpu().numpy(), o_idx)
        assert np.array_equal(res.dist.cpu().numpy().astype(np.float64), o_dist)


def test_split_deterministic_and_agrees_with_fp32_plan():
    """Two runs give the same bits.  Against the fp32 plan the lists may differ only where that
    plan's single-precision selection values cannot separate two references (this plan ranks its
    candidates on the double re-pricing): a handful of rows at most, each still the oracle's."""
    X = workloads.mixture(5000, 96, 12, seed=31)
    a, _ = _build(X, 15)
    b, _ = _build(X, 15)
    c = knn_build(X.cuda(), 15, symmetric=2, variant=3)
    torch.cuda.synchronize()
    assert torch.equal(a.idx, b.idx) and torch.equal(a.dist, b.dist)
    differ = int((a.idx != c.idx).any(dim=1).sum())
    _say(f"    rows whose list differs from the fp32 plan's: {differ} of 5000")
    assert differ <= 5
    o_idx, _, _ = oracle.build_knn(X.numpy(), 15)
    rows = (a.idx != c.idx).any(dim=1).cpu().numpy()
    assert np.array_equal(a.idx.cpu().numpy()[rows], o_idx[rows])         # where they differ, this plan has the oracle's list


def test_split_refuses_what_it_cannot_serve():
    X = workloads.gaussian(500, 300, seed=1).cuda()
    for kw, d in ((dict(metric="cosine"), 64), (dict(metric="l1"), 64), (dict(), 300)):
        with pytest.raises(api.KnnError) as e:
            knn_build(X[:, :d].contiguous(), 5, variant=SPLIT, **kw)
        assert e.value.status == api.KNN_EUNSUPPORTED
    with pytest.raises(api.KnnError) as e:
        knn_build(X[:, :64].contiguous(), 113, variant=SPLIT)
    assert e.value.status == api.KNN_EUNSUPPORTED


@pytest.mark.parametrize("which,sample,symmetric", [(1, 4096, 2), (1, 4096, 1), (2, 1024, 2), (2, 1024, 1), (3, 1024, 0),
                                                    (3, 1024, 1)])
def test_split_configs_full(which, sample, symmetric):
    """Configs 1-3 at full size, what the plan takes by itself (the full square) and each pair once: the same oracle samples and the same comparator as the fp32 plans, no exemption
    beyond theirs (0 rows)."""
    w = workloads.config(which)
    _say(f"  {w.name} split-precision symmetric={symmetric}")
    unc = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    res = knn_build(w.R.cuda(), w.k, w.metric, variant=SPLIT, symmetric=symmetric, profile=True, uncertified=unc)
    torch.cuda.synchronize()
    _say(f"    {res.plan}")
    _say(f"    gpu: {res.profile.ms_total:.1f} ms total, {res.profile.ms_main:.1f} ms main stage; "
         f"rows left unproven: {int(unc.item())} of {w.n}")
    assert int(unc.item()) == 0
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    rng = np.random.default_rng(which)
    rows = np.unique(np.concatenate([rng.choice(w.n, min(sample, w.n), replace=False),
                                     [0, 255, 256, w.n // 2, w.n - 257, w.n - 256, w.n - 1]]))
    R = w.R.numpy()
    rep = _check(R[rows], R, rows, w.k, gi[rows], gd[rows])
    assert rep.rows_set_exempt == 0
    assert np.all(np.diff(gd, axis=1) >= 0)
    assert not np.any(gi == np.arange(w.n, dtype=np.int64)[:, None])
    s = np.sort(gi, axis=1)
    assert gi.min() >= 0 and gi.max() < w.n and np.all(s[:, 1:] != s[:, :-1])
