"""rtams_search_noalloc (the entry point for callers that cannot allocate: its scratch is an array in
the library's device image) against rtams_search through the C ABI: same kernels, so the answers must
be the same bits.  Two calls in a row, the second with a smaller input (the array keeps the first
call's contents), both metrics, and the limits."""
import numpy as np
import pytest
import torch

from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import dev, make_pair
from tests.helpers import assert_topk_matches

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("metric", ["l2", "ip"])
def test_search_on_the_static_scratch_equals_search(metric):
    if metric == "l2":
        w = synth.byte_valued_l2("noalloc-l2", 91, n_base=30_000, n_centres=40, nlist=96, block_vecs=128,
                                 n_queries=200, n_inserts=64, nprobe=12, k=50)
    else:
        w = synth.unit_ip("noalloc-ip", 92, d=96, n_base=30_000, n_centres=300, nlist=128, block_vecs=256,
                          n_queries=200, n_inserts=64, nprobe=16, k=10)
    print(f"[case] {w.name} seed={w.seed}", flush=True)
    g, o = make_pair(w)
    g.add(dev(w.base)); o.add(w.base)
    s = torch.cuda.Stream()
    for mode in (1, 2):  # the default arithmetic of the scan, and the matrix cores whatever the batch
        g.set_param("scan_mfma", mode)
        for lo, nq in ((0, 64), (64, 7), (100, 1)):  # the second and third calls are smaller than the first
            q = dev(w.queries[lo:lo + nq])
            d0, i0 = g.search(q, w.k, w.nprobe, stream=s)
            s.synchronize()
            d1 = torch.full((nq, w.k), 123.0, dtype=torch.float32, device="cuda:0")
            i1 = torch.full((nq, w.k), -7, dtype=torch.int64, device="cuda:0")
            g.search_noalloc(q, w.k, w.nprobe, d1, i1, stream=s)
            s.synchronize()
            assert g.poll_error() == 0
            assert torch.equal(i0, i1) and torch.equal(d0.view(torch.int32), d1.view(torch.int32)), f"mode {mode} nq {nq}"
            rd, ri = o.search(w.queries[lo:lo + nq], w.k, w.nprobe)
            assert_topk_matches(w.metric, d1.cpu().numpy(), i1.cpu().numpy(), rd, ri, rtol=1e-4, atol=1e-6)
    g.close()


def test_limits_of_the_static_scratch():
    w = synth.gaussian_l2("noalloc-limits", 93, n_base=5_000, n_queries=128, n_inserts=10)
    g, o = make_pair(w)
    g.add(dev(w.base))
    k, nprobe = w.k, w.nprobe
    out = lambda nq: (torch.empty((nq, k), dtype=torch.float32, device="cuda:0"),
                      torch.empty((nq, k), dtype=torch.int64, device="cuda:0"))
    with pytest.raises(rtams.RtamsError) as e:  # more queries than a request on the array may hold
        g.search_noalloc(dev(w.queries[:65]), k, nprobe, *out(65))
    assert e.value.code == rtams.EINVAL and "64" in str(e.value)
    with pytest.raises(rtams.RtamsError) as e:  # the argument checks are those of rtams_search
        g.search_noalloc(dev(w.queries[:4]), 129, nprobe, torch.empty((4, 129), dtype=torch.float32, device="cuda:0"),
                         torch.empty((4, 129), dtype=torch.int64, device="cuda:0"))
    assert e.value.code == rtams.EINVAL
    # a second request before the first has finished is refused, not raced with
    s = torch.cuda.Stream()
    d1, i1 = out(64)
    refused = 0
    for _ in range(20):
        try:
            g.search_noalloc(dev(w.queries[:64]), k, nprobe, d1, i1, stream=s)
        except rtams.RtamsError as err:
            assert err.code == rtams.EBUSY
            refused += 1
    s.synchronize()
    g.search_noalloc(dev(w.queries[:64]), k, nprobe, d1, i1, stream=s)  # and accepted again once it has
    s.synchronize()
    d0, i0 = g.search(dev(w.queries[:64]), k, nprobe)
    torch.cuda.synchronize()
    assert torch.equal(i0, i1)
    g.close()
