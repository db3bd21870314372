"""Acceptance rule for a kNN answer -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Checks a candidate answer (idx, dist) against the oracle's for the same
queries.  The rule:

* every reported distance agrees with the oracle's double-precision distance
  of that (query, reference) pair within ``rtol`` relative (plus ``atol``,
  which is 0 except for degenerate inputs whose distances are ~0);
* each row is a valid Sect.-3 answer: indices distinct, in range, never the
  query itself, listed in non-decreasing order of distance (order of entries
  whose true distances differ by less than the tolerance is free);
* the neighbour SET equals the oracle's, except that entries whose oracle
  distance lies within the tolerance of the oracle's k-th distance may be
  exchanged for other references inside that same band (fp32 cannot resolve
  them); the number of rows that needed this exemption is reported.

``band_atol`` (default: ``atol``) is an absolute floor for the tie band ALONE, for distances
that can be zero or negative while their terms are not (Kullback-Leibler on un-normalised
rows): there a band relative to the k-th distance is meaningless, and the floor is derived
from the size of the terms summed (see the test that passes it).  It never loosens the check
of the reported distances.

``strict_ties=True`` drops the exemptions and demands the oracle's exact index
lists (used where the arithmetic is exact and ties go to the lower index).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import pair_dists


@dataclass
class Report:
    rows: int = 0
    ok: bool = True
    max_rel_err: float = 0.0
    rows_set_exempt: int = 0      # rows whose set differs only inside the tie band
    rows_order_exempt: int = 0    # rows listing a near-tie pair in the other order
    rows_failed: int = 0          # failures counted (the messages kept are capped)
    failures: list = field(default_factory=list)

    def fail(self, msg: str) -> None:
        self.ok = False
        self.rows_failed += 1
        if len(self.failures) < 20:
            self.failures.append(msg)

    def __str__(self) -> str:
        head = (f"rows={self.rows} ok={self.ok} max_rel_err={self.max_rel_err:.3e} "
                f"set_exempt={self.rows_set_exempt} order_exempt={self.rows_order_exempt}")
        return head + "".join("\n  " + f for f in self.failures)


def check(Q, R, metric, o_idx, o_dist, o_next, g_idx, g_dist, self_idx=None,
          rtol: float = 1e-5, atol: float = 0.0, strict_ties: bool = False,
          band_atol=None) -> Report:
    """Compare a candidate answer (g_*) with the oracle's (o_*) row by row."""
    o_idx = np.asarray(o_idx)
    o_dist = np.asarray(o_dist, dtype=np.float64)
    g_idx = np.asarray(g_idx)
    g_dist = np.asarray(g_dist, dtype=np.float64)
    nq, k = o_idx.shape
    rep = Report(rows=nq)
    if band_atol is None:
        band_atol = atol
    if g_idx.shape != (nq, k) or g_dist.shape != (nq, k):
        rep.fail(f"shape mismatch: got {g_idx.shape}/{g_dist.shape}, want {(nq, k)}")
        return rep
    nr = np.asarray(R).shape[0]
    if np.any(g_idx < 0) or np.any(g_idx >= nr):
        bad = np.argwhere((g_idx < 0) | (g_idx >= nr))[0]
        rep.fail(f"row {bad[0]} rank {bad[1]}: index {g_idx[tuple(bad)]} out of range")
        return rep
    true_d = pair_dists(Q, R, g_idx, metric)          # oracle's price of the candidate's picks

    tol = rtol * np.abs(true_d) + atol
    err = np.abs(g_dist - true_d)
    with np.errstate(divide="ignore", invalid="ignore"):
        rel = np.where(true_d != 0, err / np.abs(true_d), 0.0)
    rep.max_rel_err = float(np.max(np.where(err <= atol, 0.0, rel))) if rel.size else 0.0
    bad = np.argwhere(~(err <= tol))
    for b in bad:
        rep.fail(f"row {b[0]} rank {b[1]} idx {g_idx[tuple(b)]}: dist {g_dist[tuple(b)]!r} "
                 f"vs oracle {true_d[tuple(b)]!r}")

    if strict_ties:
        if not np.array_equal(g_idx, o_idx):
            b = np.argwhere(g_idx != o_idx)[0]
            rep.fail(f"row {b[0]}: index list {g_idx[b[0]].tolist()} != oracle {o_idx[b[0]].tolist()}")
        return rep

    for i in range(nq):
        gi = g_idx[i]
        if len(set(gi.tolist())) != k:
            rep.fail(f"row {i}: repeated index in {gi.tolist()}")
            continue
        if self_idx is not None and self_idx[i] >= 0 and int(self_idx[i]) in gi:
            rep.fail(f"row {i}: lists itself")
            continue
        td = true_d[i]
        dk = o_dist[i, k - 1]
        band = rtol * abs(dk) + band_atol
        # order: true distances non-decreasing up to the tolerance
        steps = td[1:] - td[:-1]
        if np.any(steps < -(rtol * np.abs(td[:-1]) + band_atol)):
            r = int(np.argmax(steps < -(rtol * np.abs(td[:-1]) + band_atol)))
            rep.fail(f"row {i}: order broken at rank {r}: {td[r]!r} then {td[r + 1]!r}")
            continue
        if np.any(steps < 0):
            rep.rows_order_exempt += 1
        # set
        gs, os_ = set(gi.tolist()), set(o_idx[i].tolist())
        if gs != os_:
            extra = [j for j in gi.tolist() if j not in os_]
            missing = [j for r, j in enumerate(o_idx[i].tolist()) if j not in gs]
            d_extra = td[[r for r, j in enumerate(gi.tolist()) if j not in os_]]
            d_missing = o_dist[i, [r for r, j in enumerate(o_idx[i].tolist()) if j not in gs]]
            # anything let in must sit in the band just above the k-th distance,
            # anything left out in the band just below it
            if np.all(d_extra - dk <= band) and np.all(dk - d_missing <= band) \
                    and (o_next[i] - dk <= band):
                rep.rows_set_exempt += 1
            else:
                rep.fail(f"row {i}: set differs: extra {extra} (d={d_extra.tolist()}), "
                         f"missing {missing} (d={d_missing.tolist()}), k-th {dk!r}, next {o_next[i]!r}")
    return rep
