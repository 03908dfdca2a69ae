"""Insertion and search on different streams at the same time (Multi Stream
Execution algorithm of the paper): a search must see whole insertion batches
only, i.e. its result equals the oracle's result on SOME prefix of the batches,
between those finished before it was submitted and those submitted before it
finished; at rest the results are exactly the oracle's."""
import threading

import numpy as np
import pytest
import torch

from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import assert_lists_equal, dev, make_pair
from tests.helpers import assert_topk_matches

pytestmark = pytest.mark.gpu


def matches(metric, d, i, rd, ri):
    try:
        assert_topk_matches(metric, d[None], i[None], rd[None], ri[None], rtol=1e-4, atol=1e-6)
        return True
    except AssertionError:
        return False


@pytest.mark.parametrize("n_search_threads", [1, 3])
def test_search_sees_whole_batches_only(n_search_threads):
    w = synth.gaussian_l2("concurrent", 77, n_base=10_000, n_queries=64, n_inserts=2_000, insert_batch=50,
                          nlist=64, block_vecs=64)
    g, o = make_pair(w, n_resources=8)
    g.add(dev(w.base)); o.add(w.base)
    nb = len(w.inserts) // w.insert_batch
    batches = [w.inserts[b * w.insert_batch:(b + 1) * w.insert_batch] for b in range(nb)]
    # the queries are the inserted vectors themselves, so every batch changes some answers
    qh = np.concatenate([b[:2] for b in batches])[:64]
    expected = [o.search(qh, w.k, w.nprobe)]
    for b in batches:
        o.add(b)
        expected.append(o.search(qh, w.k, w.nprobe))
    dbatches = [dev(b) for b in batches]
    q = dev(qh)
    torch.cuda.synchronize()

    data = torch.cuda.Stream()
    events = [torch.cuda.Event() for _ in range(nb)]
    started, recorded = [0], [0]        # batches whose add has begun / whose event is on the stream
    bad, checked, spread = [], [0], set()

    def completed():
        c = 0
        while c < recorded[0] and events[c].query():
            c += 1
        return c

    def inserter():
        for b in range(nb):
            started[0] = b + 1
            g.add(dbatches[b], stream=data)
            events[b].record(data)
            recorded[0] = b + 1
            if b % 4 == 3:
                data.synchronize()

    def searcher():
        s = torch.cuda.Stream()
        od = torch.empty((len(qh), w.k), dtype=torch.float32, device="cuda:0")
        oi = torch.empty((len(qh), w.k), dtype=torch.int64, device="cuda:0")
        while True:
            lo = completed()
            try:
                g.search(q, w.k, w.nprobe, od, oi, stream=s)
            except rtams.RtamsError as e:
                if e.code == rtams.EBUSY:
                    s.synchronize(); continue
                bad.append(str(e)); return
            s.synchronize()
            hi = started[0]
            d, i = od.cpu().numpy(), oi.cpu().numpy()
            for r in range(len(qh)):
                ok = [p for p in range(lo, hi + 1) if matches("l2", d[r], i[r], expected[p][0][r], expected[p][1][r])]
                if not ok:
                    bad.append(f"query {r}: no batch prefix in [{lo}, {hi}] explains the result"); return
            spread.add((lo, hi))
            checked[0] += 1
            if lo >= nb:
                return

    ts = [threading.Thread(target=searcher) for _ in range(n_search_threads)]
    ti = threading.Thread(target=inserter)
    for t in ts:
        t.start()
    ti.start()
    ti.join()
    for t in ts:
        t.join()
    assert not bad, bad[0]
    assert checked[0] >= n_search_threads
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    g.validate()
    assert_lists_equal(g, o)
    d, i = g.search(q, w.k, w.nprobe)                   # at rest: exactly the last prefix
    assert_topk_matches("l2", d.cpu().numpy(), i.cpu().numpy(), expected[-1][0], expected[-1][1], rtol=1e-4, atol=1e-6)
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
