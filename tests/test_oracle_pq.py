"""Pins of the oracle's product-quantised lists (no GPU): what the textbook
method fixes, checked against definitions written out independently here."""
import numpy as np
import pytest

from oracle.oracle import OracleIndex


def _index(d, nlist, metric, cb, centroids, T=64):
    o = OracleIndex(d, nlist, metric, T, pool_blocks=4096)
    o.set_centroids(centroids)
    o.set_codebooks(cb)
    return o


def test_lossless_quantiser_reproduces_flat_search():
    """One dimension per sub-space and a codebook that holds every byte value: byte-valued
    vectors are coded without loss, so the quantised index must answer exactly like the flat one."""
    rng = np.random.default_rng(1)
    d, nlist, n = 8, 6, 3000
    C = rng.integers(0, 256, (nlist, d)).astype(np.float32)
    x = rng.integers(0, 256, (n, d)).astype(np.float32)
    q = rng.integers(0, 256, (40, d)).astype(np.float32)
    cb = np.tile(np.arange(256, dtype=np.float32)[None, :, None], (d, 1, 1))
    for metric in ("l2", "ip"):
        flat = OracleIndex(d, nlist, metric, 64, pool_blocks=4096)
        flat.set_centroids(C)
        flat.add(x)
        pq = _index(d, nlist, metric, cb, C)
        pq.add(x)
        assert np.array_equal(pq.pq_encode(x), x.astype(np.uint8))
        fd, fi = flat.search(q, 20, 3)
        pd, pi = pq.search(q, 20, 3)
        assert np.array_equal(fi, pi) and np.array_equal(fd, pd)


@pytest.mark.parametrize("metric", ["l2", "ip"])
def test_scores_are_those_of_the_reconstruction(metric):
    """The score of a coded vector is the score of its reconstruction (the concatenation of the
    codebook entries its codes name): brute force over reconstructions gives the same top-k."""
    rng = np.random.default_rng(2)
    d, M, nlist, n = 12, 4, 5, 800
    ds = d // M
    cb = rng.standard_normal((M, 256, ds)).astype(np.float32)
    C = rng.standard_normal((nlist, d)).astype(np.float32)
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((25, d)).astype(np.float32)
    o = _index(d, nlist, metric, cb, C)
    o.add(x)
    codes = o.pq_encode(x)
    recon = np.concatenate([cb[m, codes[:, m]] for m in range(M)], axis=1).astype(np.float64)
    k = 10
    dist, ids = o.search(q, k, nlist)  # every list probed
    for i in range(len(q)):
        qq = q[i].astype(np.float64)
        s = ((recon - qq) ** 2).sum(1) if metric == "l2" else recon @ qq
        order = np.lexsort((np.arange(n), s if metric == "l2" else -s))[:k]
        assert np.allclose(dist[i], s[order], rtol=1e-12, atol=1e-12)
        # ids agree wherever the scores are not tied to the last bit
        same = ids[i] == order
        assert same.all() or np.allclose(s[ids[i][~same]], s[order[~same]], rtol=1e-12, atol=1e-12)


def test_codes_minimise_the_sub_space_distance_with_ties_to_the_lowest_entry():
    """Integer-valued data and codebooks: every distance is exact in any arithmetic, so the code
    must be numpy's first arg-min."""
    rng = np.random.default_rng(3)
    d, M = 6, 3
    ds = d // M
    cb = rng.integers(-4, 5, (M, 256, ds)).astype(np.float32)  # many duplicate entries: ties
    C = rng.integers(-4, 5, (2, d)).astype(np.float32)
    x = rng.integers(-6, 7, (500, d)).astype(np.float32)
    o = _index(d, 2, "l2", cb, C)
    codes = o.pq_encode(x)
    for m in range(M):
        sub = x[:, m * ds:(m + 1) * ds].astype(np.float64)
        dist = ((sub[:, None, :] - cb[m][None, :, :].astype(np.float64)) ** 2).sum(2)
        assert np.array_equal(codes[:, m], dist.argmin(1).astype(np.uint8))


def test_lists_hold_the_codes_in_insertion_order_and_blocks_follow_the_same_arithmetic():
    rng = np.random.default_rng(4)
    d, M, nlist, T = 8, 2, 3, 64
    cb = rng.standard_normal((M, 256, d // M)).astype(np.float32)
    C = rng.standard_normal((nlist, d)).astype(np.float32)
    x = rng.standard_normal((700, d)).astype(np.float32)
    o = _index(d, nlist, "l2", cb, C, T)
    o.add(x[:300])
    o.add(x[300:])
    a = o.assign(x)
    codes = o.pq_encode(x)
    for k in range(nlist):
        ids, lc = o.list_export_codes(k)
        assert np.array_equal(ids, np.nonzero(a == k)[0])
        assert np.array_equal(lc, codes[a == k])
        assert o.list_blocks(k) == (len(ids) + T - 1) // T
