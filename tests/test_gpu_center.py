"""knn_options_t.center: squared Euclidean distances of data far from the origin.

The expanded form |q|^2 + |r|^2 - 2 q.r loses, in fp32, about |x|^2 * 2^-23 of every distance;
for rows at 100 +- 1 per coordinate that is as much as neighbouring distances differ, and the
candidates kept are no longer the nearest.  With the column means subtracted first the same
data must pass the ordinary acceptance rule against the CPU oracle (which works in double on the
original rows) under every plan.  The rows failing without the option are printed, not judged.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import compare
from paper_0906_0231_amd import api, knn_build, knn_search

pytestmark = pytest.mark.gpu
RTOL = 1e-5


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the GPU"
    api.load_library()


def _offset_rows(n, d, seed, offset=100.0):
    g = torch.Generator().manual_seed(seed)
    return (offset + torch.randn(n, d, generator=g, dtype=torch.float32)).contiguous()


def _report(Q, R, self_idx, k, g_idx, g_dist):
    o_idx, o_dist, o_next = oracle.search(Q, R, k, "sqeuclidean", self_idx=self_idx)
    return compare.check(Q, R, "sqeuclidean", o_idx, o_dist, o_next, g_idx, g_dist, self_idx=self_idx, rtol=RTOL)


@pytest.mark.parametrize("variant", [0, 1, 3, 4, 6])
@pytest.mark.parametrize("n,d,k", [(3000, 256, 10), (2500, 20, 7), (1500, 300, 5)])
def test_build_offset_data(variant, n, d, k):
    if variant == 6 and d > 256:
        pytest.skip("the split-precision plan serves d <= 256")
    X = _offset_rows(n, d, 7 * n + d)
    Xg = X.cuda()
    res = knn_build(Xg, k, variant=variant, center=True)
    torch.cuda.synchronize()
    _say(f"  n={n} d={d} k={k} plan={res.plan.plan} kernel={res.plan.kernel.decode()}")
    rep = _report(X.numpy(), X.numpy(), np.arange(n), k, res.idx.cpu().numpy(), res.dist.cpu().numpy())
    _say(f"    centred:   {rep}")
    assert rep.ok, str(rep)
    plain = knn_build(Xg, k, variant=variant)
    torch.cuda.synchronize()
    rep0 = _report(X.numpy(), X.numpy(), np.arange(n), k, plain.idx.cpu().numpy(), plain.dist.cpu().numpy())
    _say(f"    uncentred: rows failed {rep0.rows_failed} of {n}")


@pytest.mark.parametrize("variant", [0, 1, 3, 4])
def test_search_offset_data(variant):
    """The means come from the references alone and are applied to both sides."""
    nq, nr, d, k = 700, 4000, 128, 9
    R = _offset_rows(nr, d, 11, offset=-250.0)
    Q = _offset_rows(nq, d, 12, offset=-250.0)
    res = knn_search(Q.cuda(), R.cuda(), k, variant=variant, center=True)
    torch.cuda.synchronize()
    rep = _report(Q.numpy(), R.numpy(), None, k, res.idx.cpu().numpy(), res.dist.cpu().numpy())
    _say(f"    {rep}")
    assert rep.ok, str(rep)


def test_search_offset_data_with_self_offset():
    nr, d, k, off, nq = 3000, 64, 6, 1000, 500
    R = _offset_rows(nr, d, 13, offset=60.0)
    Q = R[off:off + nq].contiguous()
    res = knn_search(Q.cuda(), R.cuda(), k, self_offset=off, center=True)
    torch.cuda.synchronize()
    rep = _report(Q.numpy(), R.numpy(), np.arange(nq) + off, k, res.idx.cpu().numpy(), res.dist.cpu().numpy())
    _say(f"    {rep}")
    assert rep.ok, str(rep)


def test_center_with_the_panel_walk():
    """Walked by pairs of row panels (thresholds in the centred p-space on both sides)."""
    n, d, k = 2600, 96, 12
    X = _offset_rows(n, d, 77, offset=150.0)
    res = knn_build(X.cuda(), k, variant=4, block_rows=768, center=True, profile=True)
    torch.cuda.synchronize()
    assert res.profile.two_phase == 2
    rep = _report(X.numpy(), X.numpy(), np.arange(n), k, res.idx.cpu().numpy(), res.dist.cpu().numpy())
    _say(f"    {rep}")
    assert rep.ok, str(rep)


def test_center_is_exact_on_a_shifted_lattice():
    """Integers 5000 .. 6999 on a line: the mean (5999.5) and every centred value are exact in
    fp32, so the answer is the lattice's, ties to the lower index, bit for bit."""
    n, k = 2000, 6
    X = (5000 + torch.arange(n, dtype=torch.float32))[:, None].contiguous()
    res = knn_build(X.cuda(), k, center=True)
    torch.cuda.synchronize()
    gi, gd = res.idx.cpu().numpy(), res.dist.cpu().numpy()
    assert gi[1000].tolist() == [999, 1001, 998, 1002, 997, 1003]
    assert gd[1000].tolist() == [1, 1, 4, 4, 9, 9]
    o_idx, o_dist, o_next = oracle.search(X.numpy(), X.numpy(), k, "sqeuclidean", self_idx=np.arange(n))
    rep = compare.check(X.numpy(), X.numpy(), "sqeuclidean", o_idx, o_dist, o_next, gi, gd,
                        self_idx=np.arange(n), rtol=RTOL, strict_ties=True)
    assert rep.ok, str(rep)


@pytest.mark.parametrize("metric", ["cosine", "l1", "hellinger", "kl"])
def test_center_ignored_for_other_distances(metric):
    """A translation changes these distances (or they do not use the expanded form): the option
    must leave the answer bit for bit what it is without it."""
    g = torch.Generator().manual_seed(5)
    X = (torch.rand(1500, 48, generator=g, dtype=torch.float32) + 0.5).cuda()
    a = knn_build(X, 8, metric=metric)
    b = knn_build(X, 8, metric=metric, center=True)
    torch.cuda.synchronize()
    assert torch.equal(a.idx, b.idx) and torch.equal(a.dist, b.dist)
    assert api.knn_workspace_bytes(1500, 1500, 48, 8, metric, symmetric=True, center=True) == \
        api.knn_workspace_bytes(1500, 1500, 48, 8, metric, symmetric=True)
