"""Pins of the CPU oracle's search against things that are not the oracle:
brute-force exact k-NN, restriction to independently recomputed probed lists,
a textbook identity between the two metrics, and an exact-rational emulation of
the fixed coarse arithmetic."""
import numpy as np
import pytest

from oracle.oracle import OracleIndex
from paper_2408_02937_amd import synth
from tests.helpers import (assert_topk_matches, brute_force_scores, brute_force_topk,
                           fma_chain_exact, order_by_score_then_id)


def build(w, n=None, ids=None):
    ix = OracleIndex(w.d, w.nlist, w.metric, w.block_vecs)
    ix.set_centroids(w.centroids)
    base = w.base if n is None else w.base[:n]
    ix.add(base, ids)
    return ix, base


@pytest.fixture(scope="module")
def tiny():
    w = synth.config(1)
    ix, base = build(w)
    return w, ix, base


def test_all_lists_probed_equals_brute_force_config1(tiny):
    """IVF with nprobe = nlist is exhaustive search (introduction: only the
    probed lists are scanned, so probing all of them scans everything)."""
    w, ix, base = tiny
    q = w.queries[:200]
    d, i = ix.search(q, w.k, w.nlist)
    ids = np.arange(len(base), dtype=np.int64)
    for r in range(len(q)):
        bd, bi = brute_force_topk("l2", base, ids, q[r], w.k)
        assert_topk_matches("l2", d[r:r + 1], i[r:r + 1], bd[None], bi[None], rtol=1e-12,
                            what=f"query {r}")


@pytest.mark.parametrize("metric", ["l2", "ip"])
@pytest.mark.parametrize("d,n,nlist,k", [(4, 50, 3, 1), (4, 300, 7, 10), (32, 2000, 16, 10),
                                         (32, 40, 8, 45)])
def test_all_lists_probed_equals_brute_force_random(metric, d, n, nlist, k):
    rng = np.random.default_rng(1000 + d + n + k)
    X = rng.standard_normal((n, d), dtype=np.float32)
    C = X[rng.permutation(n)[:nlist]].copy()
    Q = rng.standard_normal((20, d), dtype=np.float32)
    ids = rng.permutation(10 * n)[:n].astype(np.int64)          # caller-supplied ids
    ix = OracleIndex(d, nlist, metric, 4)
    ix.set_centroids(C)
    ix.add(X, ids)
    dist, got = ix.search(Q, k, nlist)
    for r in range(len(Q)):
        bd, bi = brute_force_topk(metric, X, ids, Q[r], k)       # k > n pads with -1 / inf
        assert_topk_matches(metric, dist[r:r + 1], got[r:r + 1], bd[None], bi[None], rtol=1e-12)


def test_integer_valued_data_is_exact():
    """On byte-valued data every product and partial sum is an integer below
    2^53, so the oracle must equal brute force bit for bit, ties by id included."""
    w = synth.byte_valued_l2("t", 7, d=128, n_base=3000, n_centres=20, nlist=16, block_vecs=128,
                             n_queries=30, n_inserts=10)
    # duplicate some rows so that exact ties exist
    base = np.concatenate([w.base, w.base[:200]])
    ix = OracleIndex(w.d, w.nlist, "l2", w.block_vecs)
    ix.set_centroids(w.centroids)
    ix.add(base)
    ids = np.arange(len(base), dtype=np.int64)
    d, i = ix.search(w.queries, 100, w.nlist)
    for r in range(len(w.queries)):
        bd, bi = brute_force_topk("l2", base, ids, w.queries[r], 100)
        assert np.array_equal(d[r], bd) and np.array_equal(i[r], bi)
    # a query equal to a duplicated base row must return both copies first, lower id first
    d, i = ix.search(base[5:6], 2, w.nlist)
    assert d[0, 0] == 0.0 and d[0, 1] == 0.0 and i[0].tolist() == [5, 3005]


@pytest.mark.parametrize("metric,maker", [("l2", synth.gaussian_l2), ("ip", synth.unit_ip)])
def test_partial_probe_is_brute_force_on_probed_lists(metric, maker):
    """With nprobe < nlist the answer is exact k-NN restricted to the union of
    the probed lists, where membership and probe choice are recomputed here."""
    w = maker("t", 11, n_base=4000, nlist=32, n_queries=60, n_inserts=10, block_vecs=64) \
        if metric == "l2" else maker("t", 11, d=24, n_base=4000, n_centres=50, nlist=32,
                                     n_queries=60, n_inserts=10, block_vecs=64)
    ix, base = build(w)
    ids = np.arange(len(base), dtype=np.int64)
    member = np.empty(len(base), dtype=np.int64)
    for r in range(len(base)):
        s = brute_force_scores(metric, w.centroids, base[r])
        o = order_by_score_then_id(metric, s, np.arange(w.nlist))
        member[r] = o[0]
        gap = abs(s[o[1]] - s[o[0]])
        assert gap > 1e-9 * max(1.0, abs(s[o[0]])), "generator produced a coarse near-tie"
    nprobe, k = 5, 10
    dist, got = ix.search(w.queries, k, nprobe)
    probes = ix.probe(w.queries, nprobe)
    for r in range(len(w.queries)):
        s = brute_force_scores(metric, w.centroids, w.queries[r])
        o = order_by_score_then_id(metric, s, np.arange(w.nlist))
        assert probes[r].tolist() == o[:nprobe].tolist()
        sel = np.isin(member, o[:nprobe])
        bd, bi = brute_force_topk(metric, base[sel], ids[sel], w.queries[r], k)
        assert_topk_matches(metric, dist[r:r + 1], got[r:r + 1], bd[None], bi[None], rtol=1e-12)


def test_recall_is_monotone_in_nprobe(tiny):
    w, ix, base = tiny
    q = w.queries[:100]
    _, exact = ix.search(q, w.k, w.nlist)
    last = -1.0
    for nprobe in (1, 2, 4, 8, 16, 32, 64):
        _, got = ix.search(q, w.k, nprobe)
        rec = np.mean([len(set(a) & set(b)) / w.k for a, b in zip(got.tolist(), exact.tolist())])
        assert rec >= last
        last = rec
    assert last == 1.0


def test_l2_and_ip_agree_on_unit_vectors():
    """||x-q||^2 = 2 - 2<x,q> for unit vectors: both metrics rank alike."""
    w = synth.unit_ip("t", 5, d=24, n_base=3000, n_centres=40, nlist=16, n_queries=40, n_inserts=1)
    a = OracleIndex(w.d, w.nlist, "ip", 64); a.set_centroids(w.centroids); a.add(w.base)
    b = OracleIndex(w.d, w.nlist, "l2", 64); b.set_centroids(w.centroids); b.add(w.base)
    dip, iip = a.search(w.queries, 10, w.nlist)
    dl2, il2 = b.search(w.queries, 10, w.nlist)
    assert np.allclose(dl2, 2.0 - 2.0 * dip, atol=1e-6)
    assert_topk_matches("l2", 2.0 - 2.0 * dip, iip, dl2, il2, rtol=0, atol=1e-6)


@pytest.mark.parametrize("metric", ["l2", "ip"])
def test_coarse_arithmetic_is_one_fma_per_dimension_in_order(metric):
    """The coarse score must be the fma chain bit for bit; the test looks for
    inputs where an unfused or reordered sum would differ, so that a wrong
    arithmetic is caught."""
    rng = np.random.default_rng(3)
    d, nlist = 24, 32
    C = rng.standard_normal((nlist, d), dtype=np.float32)
    ix = OracleIndex(d, nlist, metric, 4)
    ix.set_centroids(C)
    differs_from_unfused = differs_from_reversed = 0
    for _ in range(20):
        y = rng.standard_normal(d, dtype=np.float32)
        got = ix.coarse_scores(y)
        for c in range(nlist):
            assert got[c] == fma_chain_exact(metric, y, C[c])
            y64, c64 = y.astype(np.float64), C[c].astype(np.float64)
            acc = 0.0
            for j in range(d):
                acc = acc + ((y64[j] - c64[j]) ** 2 if metric == "l2" else y64[j] * c64[j])
            differs_from_unfused += acc != got[c]
            differs_from_reversed += fma_chain_exact(metric, y[::-1], C[c][::-1]) != got[c]
    # (a product of two floats is exact in double, so fusing only matters for L2)
    assert differs_from_reversed > 0 and (metric == "ip" or differs_from_unfused > 0)


def test_ranking_uses_the_double_scores_not_their_float_roundings():
    """x1 = (1 + 2^-23, 0) and x2 = (1, 2^-11) against q = 0: the squared distances
    1 + 2^-22 + 2^-46 and 1 + 2^-22 differ in double and are one number in float.
    x2 is nearer although its id is the larger one."""
    ix = OracleIndex(2, 1, "l2", 4)
    ix.set_centroids(np.zeros((1, 2), np.float32))
    x = np.array([[1 + 2.0 ** -23, 0], [1, 2.0 ** -11]], dtype=np.float32)
    ix.add(x)
    d, i = ix.search(np.zeros((1, 2), np.float32), 2, 1)
    assert i[0].tolist() == [1, 0]
    assert d[0].tolist() == [1 + 2.0 ** -22, 1 + 2.0 ** -22 + 2.0 ** -46]
    assert np.float32(d[0, 0]) == np.float32(d[0, 1])


def test_short_lists_pad_and_argument_errors():
    from oracle.oracle import OracleError
    ix = OracleIndex(4, 4, "ip", 2)
    with pytest.raises(OracleError):
        ix.search(np.zeros((1, 4), np.float32), 1, 1)           # no centroids yet
    ix.set_centroids(np.eye(4, dtype=np.float32))
    d, i = ix.search(np.ones((1, 4), np.float32), 3, 4)         # empty index
    assert np.all(i == -1) and np.all(d == -np.inf)
    ix.add(np.eye(4, dtype=np.float32)[:2])
    d, i = ix.search(np.array([[1, 0, 0, 0]], np.float32), 3, 4)
    assert i[0].tolist() == [0, 1, -1] and d[0].tolist() == [1.0, 0.0, -np.inf]
    with pytest.raises(OracleError):
        ix.search(np.zeros((1, 4), np.float32), 1, 5)           # nprobe > nlist
