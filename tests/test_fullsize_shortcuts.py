"""The shortcuts the full-size parity tests use in front of the oracle, checked on the CPU against
the oracle's own assignment on every row of small sets (both metrics, with duplicated centroids and
vectors that are centroids, where several centroids tie and the lowest index has to win), and the
threaded generator of large sets (a pure function of the seed)."""
import numpy as np
import pytest

from oracle.oracle import OracleIndex
from paper_2408_02937_amd import synth
from tests.fullsize_common import check_assignment_on_sample, filtered_assignment


@pytest.mark.parametrize("metric", ["l2", "ip"])
def test_filtered_assignment_is_the_oracle_s(metric):
    maker = synth.gaussian_l2 if metric == "l2" else synth.unit_ip
    w = maker("t", 11, d=24, n_base=6000, n_centres=60, nlist=48, n_queries=1, n_inserts=1)
    C = w.centroids.copy()
    C[17] = C[5]          # two centroids tie for every vector: the lower index takes them
    C[40] = C[41] + 1e-7  # a near tie that only the oracle's arithmetic can decide
    o = OracleIndex(w.d, w.nlist, metric, 64, pool_blocks=1)
    o.set_centroids(C)
    X = np.concatenate([w.base, C[:8]])  # some vectors are centroids themselves
    got = filtered_assignment(o, metric, X, C, rows_per_step=1000)
    assert np.array_equal(got, o.assign(X))
    assert not np.any(got == 17)
    assert check_assignment_on_sample(o, X, got, 500, seed=1) == 500


def test_a_wrong_shortcut_is_caught_by_the_sample():
    w = synth.gaussian_l2("t", 12, d=16, n_base=2000, n_centres=20, nlist=16, n_queries=1, n_inserts=1)
    o = OracleIndex(w.d, w.nlist, "l2", 64, pool_blocks=1)
    o.set_centroids(w.centroids)
    a = o.assign(w.base)
    a[::50] = (a[::50] + 1) % w.nlist
    with pytest.raises(AssertionError):
        check_assignment_on_sample(o, w.base, a, 1000, seed=2)


def test_skewed_set_by_construction_assignment_is_the_oracle_s():
    w = synth.skewed_l2("t", 13, d=64, n_base=4000, nlist=128, n_queries=1, n_inserts=1)
    o = OracleIndex(w.d, w.nlist, "l2", 64, pool_blocks=1)
    o.set_centroids(w.centroids)
    assert np.array_equal(o.assign(w.base), w.extra["base_component"])


def test_large_sets_are_a_pure_function_of_the_seed(monkeypatch):
    monkeypatch.setattr(synth, "_BIG_SET", 1 << 12)
    monkeypatch.setattr(synth, "_CHUNK_ROWS", 100)
    a = synth.unit_ip("t", 14, d=16, n_base=1000, n_centres=10, nlist=8, n_queries=300, n_inserts=10)
    monkeypatch.setattr(synth.os, "cpu_count", lambda: 1)
    b = synth.unit_ip("t", 14, d=16, n_base=1000, n_centres=10, nlist=8, n_queries=300, n_inserts=10)
    assert np.array_equal(a.base, b.base) and np.array_equal(a.queries, b.queries)
    assert np.allclose(np.linalg.norm(a.base, axis=1), 1.0, atol=1e-6)
    assert len(np.unique(a.base[:, 0])) > 900  # chunks do not repeat each other
