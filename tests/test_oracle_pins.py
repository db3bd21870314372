"""Pins for the CPU oracle: it is checked against things other than itself.

Each test names what it pins.  Citations are to the paper's sections:
Sect. 3 (problem statement: ordered k nearest, every left-out vector at least as
far as the k-th), Sect. 3 (delta symmetric, computed coordinate by coordinate),
Sect. 4 (only pairs x > y are ever evaluated, so a vector is not its own
neighbour), Sect. 7 Eq. 1 (Hellinger distance).
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import compare

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    sec, out, cur = None, {"points": [], "idx": [], "dist": [], "next": []}, None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] in ("d", "k"):
                out[tok[0]] = int(tok[1])
            elif tok[0] == "metric":
                out["metric"] = tok[1]
            elif tok[0] in out and len(tok) == 1:
                cur = tok[0]
            else:
                out[cur].append([float(t) for t in tok])
    return out


@pytest.mark.parametrize("name", ["hand_sqeuclidean.txt", "hand_cosine.txt", "hand_l1.txt",
                                  "hand_linf.txt", "hand_kl.txt"])
def test_hand_examples(name):
    """Hand-computed tables: distance formula, order, lower-index ties, self-exclusion."""
    g = _read_golden(name)
    X = np.array(g["points"], dtype=np.float32)
    idx, dist, nxt = oracle.build_knn(X, g["k"], g["metric"])
    assert idx.tolist() == [[int(v) for v in row] for row in g["idx"]]
    np.testing.assert_allclose(dist, np.array(g["dist"]), rtol=1e-15, atol=0)
    np.testing.assert_allclose(nxt, np.array(g["next"][0]), rtol=1e-15, atol=0)


def _naive_knn(Q, R, k, metric, self_idx):
    """Independent O(nq nr d) triple loop with selection by repeated minimum."""
    out_i, out_d = [], []
    for i in range(len(Q)):
        row = []
        for j in range(len(R)):
            if self_idx is not None and self_idx[i] == j:
                row.append(None)
                continue
            if metric == "sqeuclidean":
                acc = 0.0
                for c in range(len(Q[i])):
                    acc += (float(Q[i][c]) - float(R[j][c])) ** 2
            elif metric == "cosine":
                uv = uu = vv = 0.0
                for c in range(len(Q[i])):
                    uv += float(Q[i][c]) * float(R[j][c])
                    uu += float(Q[i][c]) ** 2
                    vv += float(R[j][c]) ** 2
                acc = 1.0 if uu == 0 or vv == 0 else 1.0 - uv / (math.sqrt(uu) * math.sqrt(vv))
            elif metric == "hellinger":
                acc = 0.0
                for c in range(len(Q[i])):
                    acc += (math.sqrt(float(Q[i][c])) - math.sqrt(float(R[j][c]))) ** 2
            elif metric == "l1":
                acc = 0.0
                for c in range(len(Q[i])):
                    acc += abs(float(Q[i][c]) - float(R[j][c]))
            elif metric == "linf":
                acc = 0.0
                for c in range(len(Q[i])):
                    acc = max(acc, abs(float(Q[i][c]) - float(R[j][c])))
            else:
                acc = 0.0
                for c in range(len(Q[i])):
                    if float(Q[i][c]) > 0:
                        acc += float(Q[i][c]) * math.log(float(Q[i][c]) / float(R[j][c]))
            row.append(acc)
        taken, ri, rd = set(), [], []
        for _ in range(k):
            best = None
            for j, v in enumerate(row):
                if v is None or j in taken:
                    continue
                if best is None or v < row[best]:      # strict: first (lowest) index wins ties
                    best = j
            taken.add(best)
            ri.append(best)
            rd.append(row[best])
        out_i.append(ri)
        out_d.append(rd)
    return out_i, out_d


@pytest.mark.parametrize("metric", ["sqeuclidean", "cosine", "hellinger", "l1", "linf", "kl"])
@pytest.mark.parametrize("n,d,k", [(17, 3, 4), (64, 9, 7), (40, 1, 39)])
def test_against_naive_triple_loop(metric, n, d, k):
    rng = np.random.default_rng(n * 100 + d)
    X = rng.standard_normal((n, d)).astype(np.float32)
    if metric == "hellinger":
        X = np.abs(X)
    if metric == "kl":
        X = np.abs(X) + np.float32(0.5)          # rounding below must not produce a zero reference
    # duplicate a row and quantise a few so that exact ties occur
    X[5] = X[2]
    X[7:12] = np.round(X[7:12])
    idx, dist, _ = oracle.build_knn(X, k, metric)
    ni, nd = _naive_knn(X, X, k, metric, list(range(n)))
    assert idx.tolist() == ni
    np.testing.assert_allclose(dist, np.array(nd), rtol=1e-14, atol=1e-300)


def test_query_reference_form_and_self_idx():
    """Q != R, nq != nr (a transposed operand or swapped size would break this);
    with self_idx None an identical reference is a neighbour at distance 0."""
    rng = np.random.default_rng(3)
    R = rng.standard_normal((50, 6)).astype(np.float32)
    Q = R[10:23].copy()
    idx, dist, _ = oracle.search(Q, R, 3, "sqeuclidean")
    assert idx[:, 0].tolist() == list(range(10, 23)) and np.all(dist[:, 0] == 0)
    ni, nd = _naive_knn(Q, R, 3, "sqeuclidean", None)
    assert idx.tolist() == ni
    idx2, dist2, _ = oracle.search(Q, R, 3, "sqeuclidean", self_idx=np.arange(10, 23))
    assert not np.any(idx2 == np.arange(10, 23)[:, None])
    ni2, _ = _naive_knn(Q, R, 3, "sqeuclidean", list(range(10, 23)))
    assert idx2.tolist() == ni2
    np.testing.assert_array_equal(idx[:, 1:], idx2[:, :2])


@pytest.mark.parametrize("metric", ["sqeuclidean", "cosine"])
def test_invariants(metric):
    """delta(v,v) = 0, symmetry (Sect. 3), and the two defining inequalities of Sect. 3
    verified by a scan over every left-out reference."""
    rng = np.random.default_rng(11)
    n, d, k = 200, 16, 9
    X = rng.standard_normal((n, d)).astype(np.float32)
    idx, dist, nxt = oracle.build_knn(X, k, metric)
    for i in range(0, n, 17):
        assert abs(oracle.delta(X[i], X[i], metric)) < 1e-15
        for j in range(0, n, 23):
            assert oracle.delta(X[i], X[j], metric) == oracle.delta(X[j], X[i], metric)
    assert np.all(np.diff(dist, axis=1) >= 0)
    assert not np.any(idx == np.arange(n)[:, None])
    for i in range(n):
        members = set(idx[i].tolist())
        assert len(members) == k
        rest = [oracle.delta(X[i], X[j], metric) for j in range(n) if j != i and j not in members]
        assert min(rest) >= dist[i, -1]
        assert min(rest) == nxt[i]
        for r in range(k):
            assert dist[i, r] == oracle.delta(X[i], X[idx[i, r]], metric)


def test_lattice_closed_form():
    """Points 0,1,2,..,n-1 on a line: neighbours of i are i-1,i+1,i-2,i+2,.. with
    squared distances 1,1,4,4,..; the lower index first; the ends truncate."""
    n, k = 300, 6
    X = np.arange(n, dtype=np.float32)[:, None]
    idx, dist, _ = oracle.build_knn(X, k, "sqeuclidean")
    for i in range(n):
        cand = sorted(((float((i - j) ** 2), j) for j in range(n) if j != i))[:k]
        assert idx[i].tolist() == [j for _, j in cand]
        assert dist[i].tolist() == [v for v, _ in cand]
    assert idx[100].tolist() == [99, 101, 98, 102, 97, 103]
    assert dist[100].tolist() == [1, 1, 4, 4, 9, 9]
    assert idx[0].tolist() == [1, 2, 3, 4, 5, 6]


def test_all_equidistant_and_duplicates():
    """One-hot rows: every distance is exactly 2 -> the k lowest other indices.
    Duplicated rows: the twin is the first neighbour at distance exactly 0."""
    n, k = 24, 5
    X = np.eye(n, dtype=np.float32)
    idx, dist, nxt = oracle.build_knn(X, k, "sqeuclidean")
    for i in range(n):
        assert idx[i].tolist() == [j for j in range(n) if j != i][:k]
    assert np.all(dist == 2.0) and np.all(nxt == 2.0)
    idxc, distc, _ = oracle.build_knn(X, k, "cosine")
    assert np.array_equal(idxc, idx) and np.all(distc == 1.0)
    rng = np.random.default_rng(5)
    Y = np.repeat(rng.standard_normal((10, 4)).astype(np.float32), 2, axis=0)
    idx, dist, _ = oracle.build_knn(Y, 3, "sqeuclidean")
    for i in range(20):
        assert idx[i, 0] == (i ^ 1) and dist[i, 0] == 0.0


def test_cosine_on_a_circle():
    """Unit vectors at angles t_j: cosine distance = 1 - cos(t_i - t_j), so the order
    of neighbours is the order of angular separation; scaling a row by a power of
    two changes nothing (exact in floating point)."""
    ang = np.array([0.0, 0.3, 0.5, 1.4, 2.0, 2.05, 3.0, 4.0, 5.5])
    X = np.stack([np.cos(ang), np.sin(ang)], axis=1).astype(np.float32)
    idx, dist, _ = oracle.build_knn(X, 3, "cosine")
    for i in range(len(ang)):
        sep = np.abs((ang - ang[i] + np.pi) % (2 * np.pi) - np.pi)
        order = [j for j in np.argsort(sep, kind="stable") if j != i][:3]
        assert idx[i].tolist() == order
        np.testing.assert_allclose(dist[i], 1 - np.cos(sep[order]), atol=2e-7)
    Xs = X * np.array([1, 2, 0.5, 4, 8, 0.25, 16, 1, 2], dtype=np.float32)[:, None]
    idx2, dist2, _ = oracle.build_knn(Xs, 3, "cosine")
    assert np.array_equal(idx, idx2)
    np.testing.assert_allclose(dist2, dist, rtol=0, atol=1e-15)
    Z = np.vstack([X, np.zeros((1, 2), dtype=np.float32)])
    _, dz, _ = oracle.build_knn(Z, len(ang), "cosine")
    assert np.all(dz[-1] == 1.0)                     # zero row: distance 1 to everything


def test_exact_invariances_sqeuclidean():
    """Integer data: translating all points, permuting coordinates, or permuting
    rows (indices map through the permutation where distances are distinct)
    leaves squared Euclidean distances exactly unchanged."""
    rng = np.random.default_rng(7)
    n, d, k = 60, 5, 8
    X = rng.integers(-50, 50, size=(n, d)).astype(np.float32)
    idx, dist, _ = oracle.build_knn(X, k, "sqeuclidean")
    idx_t, dist_t, _ = oracle.build_knn(X + np.float32(1000.0), k, "sqeuclidean")
    assert np.array_equal(idx, idx_t) and np.array_equal(dist, dist_t)
    idx_c, dist_c, _ = oracle.build_knn(X[:, ::-1].copy(), k, "sqeuclidean")
    assert np.array_equal(idx, idx_c) and np.array_equal(dist, dist_c)
    perm = rng.permutation(n)
    _, dist_p, _ = oracle.build_knn(X[perm], k, "sqeuclidean")
    assert np.array_equal(dist_p, dist[perm])


def test_hellinger_on_perfect_squares():
    """Eq. 1 of Sect. 7 with the square restored: on inputs a_c^2 it equals the squared
    Euclidean distance of the integer vectors a, exactly."""
    rng = np.random.default_rng(9)
    A = rng.integers(0, 30, size=(40, 6)).astype(np.float32)
    idx_h, dist_h, _ = oracle.build_knn(A * A, 5, "hellinger")
    idx_e, dist_e, _ = oracle.build_knn(A, 5, "sqeuclidean")
    assert np.array_equal(idx_h, idx_e) and np.array_equal(dist_h, dist_e)
    assert oracle.delta(np.array([4, 9]), np.array([1, 25]), "hellinger") == 1 + 4


@pytest.mark.parametrize("metric", ["sqeuclidean", "cosine"])
def test_against_library_routines(metric):
    """torch.cdist / normalised matmul in double + topk: a textbook route to the same
    numbers (sanity of values on a mid-sized input; ties are absent in this data)."""
    rng = np.random.default_rng(21)
    n, d, k = 700, 48, 12
    X = rng.standard_normal((n, d)).astype(np.float32)
    idx, dist, _ = oracle.build_knn(X, k, metric)
    T = torch.from_numpy(X).double()
    if metric == "sqeuclidean":
        D = torch.cdist(T, T, compute_mode="donot_use_mm_for_euclid_dist") ** 2
    else:
        Tn = T / T.norm(dim=1, keepdim=True)
        D = 1 - Tn @ Tn.T
    D.fill_diagonal_(float("inf"))
    td, ti = torch.topk(D, k, dim=1, largest=False)
    assert np.array_equal(idx, ti.numpy())
    np.testing.assert_allclose(dist, td.numpy(), rtol=1e-12)


@pytest.mark.parametrize("metric", ["l1", "linf", "kl"])
def test_fold_distances_against_library_routines(metric):
    """scipy's cityblock / chebyshev distance matrices and its elementwise x ln(x/y)
    (rel_entr), summed: independent routes to the same numbers; then a stable argsort."""
    from scipy.spatial.distance import cdist
    from scipy.special import rel_entr
    rng = np.random.default_rng(33)
    nq, nr, d, k = 60, 500, 24, 9
    R = rng.random((nr, d)).astype(np.float32) + np.float32(0.05)
    Q = rng.random((nq, d)).astype(np.float32)
    Q[3, :5] = 0                                  # zero query coordinates contribute nothing to KL
    if metric == "kl":
        D = rel_entr(Q.astype(np.float64)[:, None, :], R.astype(np.float64)[None, :, :]).sum(axis=2)
    else:
        D = cdist(Q.astype(np.float64), R.astype(np.float64),
                  "cityblock" if metric == "l1" else "chebyshev")
    order = np.argsort(D, axis=1, kind="stable")[:, :k]
    idx, dist, nxt = oracle.search(Q, R, k, metric)
    assert np.array_equal(idx, order)
    np.testing.assert_allclose(dist, np.take_along_axis(D, order, 1), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(nxt, np.sort(D, axis=1)[:, k], rtol=1e-12, atol=1e-13)


def test_fold_distances_closed_forms_and_invariants():
    """What the mathematics fixes: on 0/1 vectors L1 = squared Euclidean = Hamming and L-inf is
    0 or 1; L-inf <= L1 <= d L-inf; symmetry and the triangle inequality (both are metrics);
    KL against the uniform distribution is ln d minus the entropy, KL of a distribution with
    itself is 0, Gibbs' inequality, asymmetry, and scaling the query by s adds s ln s sum(q)."""
    from scipy.stats import entropy
    rng = np.random.default_rng(5)
    B = (rng.random((30, 12)) < 0.4).astype(np.float32)
    for i in range(0, 30, 3):
        for j in range(1, 30, 4):
            ham = float(np.sum(B[i] != B[j]))
            assert oracle.delta(B[i], B[j], "l1") == ham == oracle.delta(B[i], B[j], "sqeuclidean")
            assert oracle.delta(B[i], B[j], "linf") == (1.0 if ham > 0 else 0.0)
    X = rng.standard_normal((25, 7)).astype(np.float32)
    for m in ("l1", "linf"):
        for i in range(25):
            assert oracle.delta(X[i], X[i], m) == 0.0
            for j in range(i):
                dij = oracle.delta(X[i], X[j], m)
                assert dij == oracle.delta(X[j], X[i], m) and dij > 0
                for l in range(0, 25, 6):
                    assert dij <= oracle.delta(X[i], X[l], m) + oracle.delta(X[l], X[j], m) + 1e-12
    for i in range(25):
        for j in range(i):
            l1, li = oracle.delta(X[i], X[j], "l1"), oracle.delta(X[i], X[j], "linf")
            assert li <= l1 <= 7 * li
    assert oracle.delta(np.array([3, -4, 0.5]), np.array([1, 1, 1]), "l1") == 2 + 5 + 0.5
    assert oracle.delta(np.array([3, -4, 0.5]), np.array([1, 1, 1]), "linf") == 5
    d = 16
    P = rng.random((10, d)).astype(np.float32)
    P /= P.sum(axis=1, keepdims=True)
    P = P.astype(np.float32)
    U = np.full(d, 1.0 / d, dtype=np.float32)       # 1/16 is exact in fp32
    for i in range(10):
        p64 = P[i].astype(np.float64)
        s = p64.sum()
        # sum p ln(p d) = s ln d - H for the unnormalised entropy H = -sum p ln p
        want = s * math.log(d) + float(np.sum(p64 * np.log(p64)))
        assert abs(oracle.delta(P[i], U, "kl") - want) < 1e-14
        assert abs(oracle.delta(P[i], P[i], "kl")) == 0.0
        pn = p64 / s
        for j in range(10):
            qn = P[j].astype(np.float64) / P[j].astype(np.float64).sum()
            got = oracle.delta(pn.astype(np.float32), qn.astype(np.float32), "kl")
            if i != j:
                assert got > -1e-6                   # Gibbs (inputs are normalised only to fp32 accuracy)
            ref = entropy(pn.astype(np.float32).astype(np.float64), qn.astype(np.float32).astype(np.float64))
            # scipy normalises its arguments; ours are normalised to 1e-7, so agree to that order
            assert abs(got - ref) < 1e-5
    a, b = P[0], P[1]
    assert oracle.delta(a, b, "kl") != oracle.delta(b, a, "kl")
    two = oracle.delta((2 * a).astype(np.float32), b, "kl")
    assert abs(two - (2 * oracle.delta(a, b, "kl") + 2 * math.log(2) * float(a.astype(np.float64).sum()))) < 1e-14
    assert oracle.delta(np.array([0, 2.0]), np.array([5, 1.0]), "kl") == 2 * math.log(2)   # 0 ln 0 = 0


def test_comparator_accepts_oracle_and_catches_mistakes():
    """The acceptance rule itself: passes the oracle's own answer and fp32-rounded
    distances, fails a wrong index, a wrong distance, a broken order, a self match."""
    rng = np.random.default_rng(2)
    n, d, k = 150, 12, 6
    X = rng.standard_normal((n, d)).astype(np.float32)
    selfi = np.arange(n)
    idx, dist, nxt = oracle.build_knn(X, k)
    ok = compare.check(X, X, "sqeuclidean", idx, dist, nxt, idx, dist.astype(np.float32), selfi)
    assert ok.ok and ok.rows_set_exempt == 0, str(ok)
    bad = idx.copy(); bad[3, 2] = (idx[3, 2] + 1) % n
    if bad[3, 2] in idx[3] or bad[3, 2] == 3:
        bad[3, 2] = [j for j in range(n) if j != 3 and j not in idx[3]][0]
    assert not compare.check(X, X, "sqeuclidean", idx, dist, nxt, bad, dist, selfi).ok
    bd = dist.copy(); bd[4, 1] *= 1 + 1e-4
    assert not compare.check(X, X, "sqeuclidean", idx, dist, nxt, idx, bd, selfi).ok
    sw = idx.copy(); sw[5, [0, k - 1]] = sw[5, [k - 1, 0]]
    sd = dist.copy(); sd[5, [0, k - 1]] = sd[5, [k - 1, 0]]
    assert not compare.check(X, X, "sqeuclidean", idx, dist, nxt, sw, sd, selfi).ok
    se = idx.copy(); se[6, 0] = 6
    sed = dist.copy(); sed[6, 0] = 0
    assert not compare.check(X, X, "sqeuclidean", idx, dist, nxt, se, sed, selfi).ok
    # a near-tie at the boundary may be exchanged: build one on purpose
    Y = np.zeros((4, 2), dtype=np.float32)
    Y[1] = [1, 0]; Y[2] = [0, 1 + 2e-7]; Y[3] = [5, 5]
    oi, od, on = oracle.build_knn(Y, 1)
    gi = oi.copy(); gi[0, 0] = 2
    gd = oracle.pair_dists(Y, Y, gi)
    rep = compare.check(Y, Y, "sqeuclidean", oi, od, on, gi, gd, np.arange(4))
    assert rep.ok and rep.rows_set_exempt == 1, str(rep)
    assert not compare.check(Y, Y, "sqeuclidean", oi, od, on, gi, gd, np.arange(4),
                             strict_ties=True).ok


def test_select_pins():
    """Batched partial sort (Sect. 6): hand example with ties, numpy's stable argsort (a
    library routine), repeated minimum on a small input, rows independent of each other."""
    A = np.array([[5, 1, 4, 1, 9, 0], [2, 2, 2, 2, 2, 2], [-1, 7, -3, 7, -3, 8]], dtype=np.float32)
    idx, val = oracle.select(A, 4)
    assert idx.tolist() == [[5, 1, 3, 2], [0, 1, 2, 3], [2, 4, 0, 1]]          # worked out by hand
    assert val.tolist() == [[0, 1, 1, 4], [2, 2, 2, 2], [-3, -3, -1, 7]]
    rng = np.random.default_rng(4)
    B = np.round(rng.standard_normal((37, 501)) * 8).astype(np.float32) / 8      # many ties
    idx, val = oracle.select(B, 23)
    order = np.argsort(B, axis=1, kind="stable")[:, :23]
    assert np.array_equal(idx, order)
    assert np.array_equal(val, np.take_along_axis(B, order, axis=1))
    for i in (0, 17, 36):
        row, taken = B[i].tolist(), []
        for _ in range(23):
            best = None
            for j, v in enumerate(row):
                if j not in taken and (best is None or v < row[best]):
                    best = j
            taken.append(best)
        assert idx[i].tolist() == taken
    i2, v2 = oracle.select(B[5:6], 23)
    assert np.array_equal(i2[0], idx[5]) and np.array_equal(v2[0], val[5])
