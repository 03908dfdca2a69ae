"""Random sequences of operations (adds of all sizes, searches of all shapes,
rearrangements) on randomly shaped indexes of every kind (float, half and byte
storage, quantised lists, both metrics, either reservation order, every setting
of the matrix-core filter), each step checked against the oracle."""
import numpy as np
import pytest
import torch

from oracle.oracle import OracleIndex
from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import assert_lists_equal, dev
from tests.helpers import ATOL, ATOL_PQ, assert_topk_matches

pytestmark = pytest.mark.gpu


def shape_of(seed):
    rng = np.random.default_rng(seed)
    storage = str(rng.choice(["f32", "f32", "f16", "u8"]))
    d = int(rng.choice([16, 32, 48, 64, 96, 128]))
    pq = int(rng.choice([m for m in (4, 8, 16) if d % m == 0])) if storage == "f32" and rng.random() < 0.25 else 0
    return dict(seed=seed, storage=storage, pq=pq, d=d, metric=str(rng.choice(["l2", "ip"])),
                nlist=int(rng.choice([1, 2, 3, 17, 64, 65, 300, 1025])), T=int(rng.choice([64, 128, 256])),
                thr=int(rng.choice([0, 0, 150, 600])), n_base=int(rng.integers(0, 30000)),
                nres=int(rng.integers(1, 5)), mfma=int(rng.choice([0, 1, 2])), ordered=int(rng.random() < 0.3),
                maxadd=int(rng.choice([256, 1000, 4096, 65536])), steps=int(rng.integers(10, 30))), rng


@pytest.mark.parametrize("seed", list(range(7000, 7014)))
def test_random_operations_against_the_oracle(seed):
    c, rng = shape_of(seed)
    print(f"[case] {c}", flush=True)
    d, nlist, metric, storage, pq = c["d"], c["nlist"], c["metric"], c["storage"], c["pq"]
    centres = rng.uniform(40, 200, (max(3, nlist // 3), d))

    def draw(n):
        x = centres[rng.integers(0, len(centres), n)] + 12 * rng.standard_normal((n, d))
        if metric == "ip" and storage != "u8":
            x = x / np.linalg.norm(x, axis=1, keepdims=True)
        elif storage == "u8" or rng.random() < 0.3:
            x = np.clip(np.rint(x), 0, 255)  # byte-valued: exact ties abound
        return x.astype(np.float32)

    base = draw(c["n_base"] + max(nlist, 256))
    C = base[rng.permutation(len(base))[:nlist]].copy()
    cap = c["n_base"] + 60000
    blocks = cap // c["T"] + 2 * nlist + 16
    g = rtams.Index(d, nlist, metric, c["T"], pool_blocks=blocks, rearrange_threshold=c["thr"],
                    n_resources=c["nres"], max_batch=256, max_k=128, max_nprobe=min(64, nlist),
                    max_add_batch=c["maxadd"], candidates_per_query=cap + 64, pq_m=pq, storage=storage)
    o = OracleIndex(d, nlist, metric, c["T"], rearrange_threshold=c["thr"], pool_blocks=blocks)
    g.set_centroids(dev(C)); o.set_centroids(C)
    if storage != "f32":
        o.set_storage(storage)
    if pq:
        cb = synth.codebooks_from_rows(seed, base, pq)
        g.set_codebooks(dev(cb)); o.set_codebooks(cb)
    g.set_param("use_mfma", c["mfma"])
    g.set_param("ordered_add", c["ordered"])
    arith = np.random.default_rng(seed + 1)  # which arithmetic each search scans with (a stream of its own)
    if c["n_base"]:
        g.add(dev(base[:c["n_base"]])); o.add(base[:c["n_base"]])
    added = c["n_base"]
    for step in range(c["steps"]):
        op = rng.random()
        if op < 0.4 and added < cap - 20000:
            n = int(rng.choice([1, 63, 65, 1000, 4097, 20000]))
            y = draw(n)
            if rng.random() < 0.3:  # everything into one list
                y = np.repeat(y[:1], n, axis=0) if storage == "u8" else \
                    (y[0] + 0.5 * rng.standard_normal(y.shape)).astype(np.float32)
            g.add(dev(y)); o.add(y)
            added += n
        elif op < 0.5:
            lst = int(rng.integers(-1, nlist))
            g.rearrange(lst)
            if lst >= 0:
                o.rearrange(lst)
        else:
            nq = int(rng.choice([1, 2, 5, 8, 9, 33, 64, 200, 256]))
            k = int(rng.choice([1, 3, 10, 50, 100, 128]))
            nprobe = int(rng.integers(1, min(64, nlist) + 1))
            q = draw(nq)
            scan_mfma = int(arith.choice([0, 1, 2, 2]))
            g.set_param("scan_mfma", scan_mfma)  # dot products on the matrix cores, or on the vector unit
            dd, ii = g.search(dev(q), k, nprobe)
            torch.cuda.synchronize()
            assert g.poll_error() == 0, f"step {step}"
            rd, ri = o.search(q, k, nprobe)
            assert_topk_matches(metric, dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=1e-4,
                                atol=ATOL_PQ if pq else ATOL, what=f"step {step}: nq {nq} k {k} nprobe {nprobe} scan_mfma {scan_mfma}")
    torch.cuda.synchronize()
    g.validate()
    assert g.poll_error() == 0
    assert np.array_equal(g.list_sizes(), o.list_sizes())
    if not pq:
        assert_lists_equal(g, o)
    g.close()
