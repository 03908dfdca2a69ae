"""The shapes of configurations 3, 4 and 5 — their d, nlist, T_m, nprobe, k, metric, batch sizes
and stream counts — on base sets small enough for the oracle (its coarse assignment is nlist * d
multiply-adds per vector in double).  Lists bit for bit, searches within the tolerance, and for
configuration 5 the skewed growth with rearrangement rounds between the insertion batches."""
import threading

import numpy as np
import pytest
import torch

from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import assert_lists_equal, dev, make_pair
from tests.helpers import assert_topk_matches, RTOL

pytestmark = pytest.mark.gpu



def load(w, g, o):
    g.add(dev(w.base)); o.add(w.base)
    bounds = [len(w.base)]
    for b in range(0, len(w.inserts), w.insert_batch):
        chunk = w.inserts[b:b + w.insert_batch]
        g.add(dev(chunk)); o.add(chunk)
        bounds.append(bounds[-1] + len(chunk))
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    return np.array(bounds[:-1])


def check_search(w, g, o, q, what):
    d, i = g.search(dev(q), w.k, w.nprobe)
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    rd, ri = o.search(q, w.k, w.nprobe)
    assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6, what=what)


def test_configuration_3_shape_deep_embeddings():
    """IP on unit vectors, d = 96, nlist 4096, T_m 256, nprobe 64, k 10, query batch 128,
    4 search streams beside the insert stream."""
    w = synth.unit_ip("config3-shape", 53, d=96, n_base=100_000, n_centres=10_000, nlist=4096, block_vecs=256,
                      n_queries=1_024, n_inserts=4_096, insert_batch=512, nprobe=64, k=10)
    print(f"[case] {w.name} seed={w.seed} n={len(w.base)}", flush=True)
    g, o = make_pair(w, n_resources=8)
    bounds = load(w, g, o)
    g.validate()
    assert_lists_equal(g, o, bounds)
    check_search(w, g, o, w.queries[:128], "batch 128")
    # four search streams and the insert stream at once.  An answer reflects the batches published
    # before its scan, so the inserted vectors are made harmless: a thousandth of the length of the
    # data, their inner product with any query stays below every top-10 score, and the answers must be
    # the static oracle's whatever the interleaving.
    far = (1e-3 * w.inserts[:2048]).astype(np.float32)
    rd, ri = o.search(w.queries[:512], w.k, w.nprobe)
    streams = [torch.cuda.Stream() for _ in range(4)]
    data = torch.cuda.Stream()
    outs = []

    # inputs stay alive (and untouched) until the streams that read them have drained
    far_dev = [dev(far[b:b + 512]) for b in range(0, len(far), 512)]
    q_dev = [dev(w.queries[j * 128:(j + 1) * 128]) for j in range(4)]
    torch.cuda.synchronize()

    def inserter():
        for y in far_dev:
            g.add(y, stream=data)

    th = threading.Thread(target=inserter)
    th.start()
    for j in range(4):
        outs.append(g.search(q_dev[j], w.k, w.nprobe, stream=streams[j]))
    th.join()
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    o.add(far)
    rd2, ri2 = o.search(w.queries[:512], w.k, w.nprobe)
    assert np.array_equal(ri, ri2), "the short vectors were meant to stay out of every top-k"
    for j, (d, i) in enumerate(outs):
        assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd[j * 128:(j + 1) * 128],
                            ri[j * 128:(j + 1) * 128], rtol=RTOL, atol=1e-6, what=f"stream {j}")
    g.validate()
    assert_lists_equal(g, o)
    g.close()


def test_configuration_4_shape_wide_embeddings():
    """IP on unit vectors, d = 768, nlist 8192, T_m 128, nprobe 32, k 10, query batches 1..64."""
    w = synth.unit_ip("config4-shape", 54, d=768, n_base=16_000, n_centres=2_000, nlist=8192, block_vecs=128,
                      n_queries=256, n_inserts=1_024, insert_batch=64, nprobe=32, k=10)
    print(f"[case] {w.name} seed={w.seed} n={len(w.base)}", flush=True)
    g, o = make_pair(w, n_resources=8)
    bounds = load(w, g, o)
    g.validate()
    assert_lists_equal(g, o, bounds)
    for batch, start in ((1, 0), (7, 1), (64, 8), (64, 72)):
        check_search(w, g, o, w.queries[start:start + batch], f"batch {batch}")
    assert np.array_equal(g.probe(dev(w.queries), w.nprobe).cpu().numpy(), o.probe(w.queries, w.nprobe))
    g.close()


def test_configuration_5_shape_skewed_growth_with_rearrangement():
    """L2, d = 256, nlist 16384, T_m 256, Zipf(1.1) list popularity, nprobe 64, k 50, query batch 256;
    inserts in batches of 1024 with Exceed() armed, so rearrangement rounds run between them."""
    w = synth.skewed_l2("config5-shape", 55, d=256, n_base=40_000, nlist=16384, exponent=1.1, block_vecs=256,
                        n_queries=512, n_inserts=8_192, insert_batch=1024, nprobe=64, k=50)
    print(f"[case] {w.name} seed={w.seed} n={len(w.base)}", flush=True)
    n_all = len(w.base) + len(w.inserts)
    g, o = make_pair(w, pool_blocks=n_all // w.block_vecs + 2 * w.nlist + 512, rearrange_threshold=300,
                     n_resources=8)
    # the base set in batches too, so that the hot lists' chains interleave with everything else
    for b in range(0, len(w.base), 4096):
        g.add(dev(w.base[b:b + 4096])); o.add(w.base[b:b + 4096])
    for b in range(0, len(w.inserts), w.insert_batch):
        chunk = w.inserts[b:b + w.insert_batch]
        g.add(dev(chunk)); o.add(chunk)
        if b == 4 * w.insert_batch:
            check_search(w, g, o, w.queries[256:512], "between insertion batches")
    g.rearrange(-1)  # the rounds the last batch asked for
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    g.validate()
    assert o.n_rearrange > 0, "the workload was meant to trigger rearrangement"
    assert_lists_equal(g, o)
    sizes = g.list_sizes()
    hot = int(sizes.argmax())
    assert sizes[hot] > 4 * w.block_vecs                      # a hot list of many blocks ...
    assert g.pool_stats().lists_exceeding == 0                # ... that no longer exceeds (when its last round ran
    g.rearrange(hot)                                          # depends on when the device's report reached the host),
    assert g.list_info(hot)[1] == 1                           # and is one run once it is asked for
    g.validate()
    assert_lists_equal(g, o)
    check_search(w, g, o, w.queries[:256], "batch 256")
    g.close()
