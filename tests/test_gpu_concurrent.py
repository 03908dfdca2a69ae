"""Insertion and search on different streams at the same time (Multi Stream
Execution algorithm of the paper): a search must see whole insertion batches
only, i.e. its result equals the oracle's result on SOME prefix of the batches,
between those finished before it was submitted and those submitted before it
finished; at rest the results are exactly the oracle's."""
import pytest
import torch

from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import assert_lists_equal, dev, make_pair, whole_batches_check

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_search_threads", [1, 3])
def test_search_sees_whole_batches_only(n_search_threads):
    w = synth.gaussian_l2("concurrent", 77, n_base=10_000, n_queries=64, n_inserts=2_000, insert_batch=50,
                          nlist=64, block_vecs=64)
    g, o = make_pair(w, n_resources=8)
    whole_batches_check(w, g, o, n_search_threads)
    assert_lists_equal(g, o)
    g.close()


def test_requests_are_rejected_when_every_resource_is_in_flight():
    """The resource pool has a fixed number of slots; a request beyond them is
    refused with EBUSY and nothing is enqueued (paper, deployment detail)."""
    w = synth.gaussian_l2("busy", 78, n_base=20_000, n_queries=256, n_inserts=10, nlist=64, block_vecs=64)
    g, o = make_pair(w, n_resources=2)
    g.add(dev(w.base))
    q = dev(w.queries)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(3)]
    gate = torch.cuda.Event()
    hold = torch.cuda.Stream()
    # keep the first two requests from finishing: their streams wait for an event that is recorded later
    with torch.cuda.stream(hold):
        torch.cuda._sleep(200_000_000)                  # ~0.1 s of device time
        gate.record(hold)
    outs = []
    for s in streams[:2]:
        s.wait_event(gate)
        outs.append(g.search(q, 10, 8, stream=s))
    with pytest.raises(rtams.RtamsError) as e:
        g.search(q, 10, 8, stream=streams[2])
    assert e.value.code == rtams.EBUSY
    torch.cuda.synchronize()
    d, i = g.search(q, 10, 8, stream=streams[2])        # slots are free again
    torch.cuda.synchronize()
    assert torch.equal(i, outs[0][1]) and torch.equal(i, outs[1][1])
    g.close()
