"""Seeded random shapes against the oracle: dimensions, list counts (beyond 16,384 too: the plan of
the scan then walks the pair counters in more than one round), block sizes, probe counts, k, metrics,
ragged batches, flat and quantised lists.  Small data: each case takes the oracle a second or two."""
import numpy as np
import pytest
import torch

from oracle.oracle import OracleIndex
from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import assert_lists_equal, dev
from tests.helpers import ATOL, ATOL_PQ, assert_topk_matches

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(seed)
    metric = ["l2", "ip"][int(rng.integers(2))]
    d = int(rng.choice([4, 8, 12, 20, 32, 64, 100, 128, 260]))
    nlist = int(rng.choice([1, 3, 17, 64, 200, 1025, 5000, 20000]))
    T = int(rng.choice([64, 128, 192, 256]))
    n = int(rng.integers(2_000, 12_000))
    if nlist * d * n > 6e9:
        n = max(500, int(6e9 / (nlist * d)))
    nprobe = int(min(nlist, rng.choice([1, 2, 5, 16, 33, 64])))
    k = int(rng.choice([1, 3, 10, 50, 128]))
    pq = 0
    if d % 4 == 0 and rng.random() < 0.4:
        ms = [m for m in (4, 8, 16, 32, 64) if d % m == 0]
        if ms:
            pq = int(rng.choice(ms))
    batches = [int(b) for b in rng.choice([1, 2, 7, 31, 64, 100, 256], size=2, replace=False)]
    return dict(seed=seed, metric=metric, d=d, nlist=nlist, T=T, n=n, nprobe=nprobe, k=k, pq=pq, batches=batches)


# lists beyond 16,384 (the plan of the scan reads the pair counters in several rounds), both metrics
EXTRA = [
    dict(seed=951, metric="l2", d=8, nlist=20_000, T=64, n=30_000, nprobe=64, k=10, pq=0, batches=[256, 3]),
    dict(seed=952, metric="l2", d=16, nlist=40_000, T=128, n=9_000, nprobe=33, k=50, pq=0, batches=[100, 1]),
    dict(seed=953, metric="ip", d=8, nlist=33_000, T=64, n=20_000, nprobe=64, k=10, pq=4, batches=[256, 7]),
    dict(seed=954, metric="l2", d=128, nlist=1025, T=128, n=20_000, nprobe=64, k=128, pq=16, batches=[256, 31]),
]
CASES = [draw_case(s) for s in range(901, 913)] + EXTRA


@pytest.mark.parametrize("c", CASES, ids=[f"seed{c['seed']}" for c in CASES])
def test_random_shape(c):
    seed = c["seed"]
    print(f"[case] {c}", flush=True)
    rng = np.random.default_rng(seed + 10_000)
    d, nlist, n = c["d"], c["nlist"], c["n"]
    centres = rng.standard_normal((min(nlist, 64) + 3, d)).astype(np.float32)
    def draw(m):
        x = centres[rng.integers(len(centres), size=m)] + 0.3 * rng.standard_normal((m, d)).astype(np.float32)
        if c["metric"] == "ip":
            x /= np.maximum(np.linalg.norm(x, axis=1, keepdims=True), 1e-20)
        return np.ascontiguousarray(x.astype(np.float32))
    base, queries = draw(n), draw(256)
    cents = draw(nlist) if nlist > n else np.ascontiguousarray(base[rng.permutation(n)[:nlist]])
    pool_blocks = n // c["T"] + 2 * nlist + 16
    g = rtams.Index(d, nlist, c["metric"], c["T"], pool_blocks=pool_blocks, n_resources=2, max_batch=256,
                    max_k=128, max_nprobe=min(64, nlist), max_add_batch=4096, candidates_per_query=n + 64,
                    pq_m=c["pq"])
    o = OracleIndex(d, nlist, c["metric"], c["T"], pool_blocks=pool_blocks)
    g.set_centroids(dev(cents)); o.set_centroids(cents)
    if c["pq"]:
        cb = synth.codebooks_from_rows(seed, base, c["pq"])
        g.set_codebooks(dev(cb)); o.set_codebooks(cb)
    cut = n // 3
    for part in (base[:cut], base[cut:cut + 37], base[cut + 37:]):  # three batches, one of them small and ragged
        g.add(dev(part)); o.add(part)
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    g.validate()
    if c["pq"]:
        assert np.array_equal(g.list_sizes(), o.list_sizes())
        for lst in rng.choice(nlist, size=min(nlist, 8), replace=False):
            gi, gc = g.list_export_codes(int(lst))
            oi, oc = o.list_export_codes(int(lst))
            a, b = np.argsort(gi.cpu().numpy(), kind="stable"), np.argsort(oi, kind="stable")
            assert np.array_equal(gi.cpu().numpy()[a], oi[b]) and np.array_equal(gc.cpu().numpy()[a], oc[b])
    elif nlist <= 1100:
        assert_lists_equal(g, o)
    else:
        assert np.array_equal(g.list_sizes(), o.list_sizes())
    for bs in c["batches"]:
        q = queries[:bs]
        dd, ii = g.search(dev(q), c["k"], c["nprobe"])
        torch.cuda.synchronize()
        assert g.poll_error() == 0
        rd, ri = o.search(q, c["k"], c["nprobe"])
        assert_topk_matches(c["metric"], dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=1e-4, atol=ATOL_PQ if c.get("pq") else ATOL,
                            what=f"batch {bs}")
    g.close()
