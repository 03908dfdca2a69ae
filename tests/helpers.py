"""Checks shared by the oracle pins and the GPU parity tests.  Everything here
is independent of both implementations: plain numpy on the raw inputs."""
from __future__ import annotations

from fractions import Fraction

import numpy as np


# The tolerance of every comparison of fp32 scores with the oracle's doubles: 1e-4 relative (the figure the
# build states) plus 1e-6 absolute for scores near zero.  Scores of product-quantised lists are sums of M
# table entries, each rounded to fp32 on its own, of either sign for inner products: their absolute part
# is 1e-5.
RTOL, ATOL, ATOL_PQ = 1e-4, 1e-6, 1e-5


def brute_force_scores(metric: str, X: np.ndarray, q: np.ndarray) -> np.ndarray:
    """Exact-definition scores of one query against every row of X, in float64."""
    X64, q64 = X.astype(np.float64), q.astype(np.float64)
    if metric == "l2":
        diff = X64 - q64
        return np.einsum("ij,ij->i", diff, diff)
    return X64 @ q64


def order_by_score_then_id(metric: str, scores: np.ndarray, ids: np.ndarray) -> np.ndarray:
    key = scores if metric == "l2" else -scores
    return np.lexsort((ids, key))


def brute_force_topk(metric: str, X: np.ndarray, ids: np.ndarray, q: np.ndarray, k: int):
    """Top-k by (score, id) over all rows of X; padded with id -1 / +-inf."""
    s = brute_force_scores(metric, X, q) if len(X) else np.zeros(0)
    o = order_by_score_then_id(metric, s, ids)[:k]
    pad = k - len(o)
    bad = np.inf if metric == "l2" else -np.inf
    return (np.concatenate([s[o], np.full(pad, bad)]),
            np.concatenate([ids[o], np.full(pad, -1, dtype=np.int64)]))


def assert_topk_matches(metric, got_d, got_i, ref_d, ref_i, rtol, atol=0.0, what=""):
    """got == ref up to ties: distances agree position by position within the
    tolerance; an id may differ only where its reference distance is within TWICE
    the tolerance of the distance of the position it is compared with or of the
    k-th (boundary) distance.  (Twice: the implementation ranks by its own scores,
    each within the tolerance t of the reference; two candidates it puts the other
    way round therefore lie within 2 t of each other in the reference, and no closer
    bound holds.)"""
    got_d, ref_d = np.asarray(got_d, dtype=np.float64), np.asarray(ref_d, dtype=np.float64)
    assert got_d.shape == ref_d.shape and got_i.shape == ref_i.shape, what
    fin = np.isfinite(ref_d)
    assert np.array_equal(np.isfinite(got_d), fin), f"{what}: padding differs"
    assert np.array_equal(got_d[~fin], ref_d[~fin]), f"{what}: padding value differs"
    assert np.array_equal(got_i[~fin], ref_i[~fin]), f"{what}: padding ids differ"
    tol = atol + rtol * np.abs(ref_d[fin])
    err = np.abs(got_d[fin] - ref_d[fin])
    assert np.all(err <= tol), f"{what}: distance error {err.max()} beyond tolerance"
    nq, k = ref_i.shape
    for r in range(nq):
        if np.array_equal(got_i[r], ref_i[r]):
            continue
        nfin = int(fin[r].sum())
        g, f = got_i[r, :nfin], ref_i[r, :nfin]
        assert len(set(g.tolist())) == nfin, f"{what}: query {r} returns an id twice"
        dref = dict(zip(f.tolist(), ref_d[r, :nfin].tolist()))
        kth = ref_d[r, nfin - 1]
        t_k = atol + rtol * abs(kth)
        for pos in range(nfin):
            if g[pos] == f[pos]:
                continue
            # the id the reference has here must be tied with what we got
            dg = got_d[r, pos]
            t = atol + rtol * abs(ref_d[r, pos])
            if g[pos] in dref:
                assert abs(dref[int(g[pos])] - ref_d[r, pos]) <= 2 * t, \
                    f"{what}: query {r} pos {pos}: order differs beyond a tie"
            else:
                # not in the reference top-k at all: only legal as a tie at the boundary
                assert abs(dg - kth) <= 2 * t_k, \
                    f"{what}: query {r} pos {pos}: id {g[pos]} is not a boundary tie"


def fma_chain_exact(metric: str, y: np.ndarray, c: np.ndarray) -> float:
    """The fixed coarse arithmetic, emulated with exact rationals: every step is
    round_to_double(exact(a*b + acc)), which is what a fused multiply-add does."""
    acc = Fraction(0)
    for yj, cj in zip(y.tolist(), c.tolist()):
        if metric == "l2":
            t = Fraction(float(Fraction(yj) - Fraction(cj)))  # double subtraction, rounded once
            acc = Fraction(float(t * t + acc))
        else:
            acc = Fraction(float(Fraction(yj) * Fraction(cj) + acc))
    return float(acc)


def canonical_lists(ids_per_list, vecs_per_list):
    """Sort every list's content by id so two indexes can be compared as sets."""
    out = []
    for ids, x in zip(ids_per_list, vecs_per_list):
        o = np.argsort(ids, kind="stable")
        out.append((ids[o], x[o]))
    return out
