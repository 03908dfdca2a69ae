"""The scratch reserve shared by all stream resources (the paper's overflow chunks
from a central pool, Deployment Detail): a request whose candidates do not fit
into its resource's own slice leases a chunk there and returns it."""
import threading

import numpy as np
import pytest
import torch

from oracle.oracle import OracleIndex
from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import dev
from tests.helpers import assert_topk_matches, RTOL

pytestmark = pytest.mark.gpu



def small_set():
    return synth.byte_valued_l2("byte-overflow", 31, n_base=30_000, n_centres=40, nlist=96, block_vecs=128,
                                n_queries=512, n_inserts=64, insert_batch=64, nprobe=12, k=100)


def build(w, candidates_per_query, overflow_candidates, pq_m=0, n_resources=4, overflow_chunks=4):
    g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=len(w.base) // w.block_vecs + 2 * w.nlist,
                    n_resources=n_resources, max_batch=64, max_k=128, max_nprobe=16,
                    candidates_per_query=candidates_per_query, overflow_candidates=overflow_candidates,
                    overflow_chunks=overflow_chunks, pq_m=pq_m)
    o = OracleIndex(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=len(w.base) // w.block_vecs + 2 * w.nlist)
    g.set_centroids(dev(w.centroids))
    o.set_centroids(w.centroids)
    if pq_m:
        cb = synth.codebooks_from_rows(w.seed, w.base, pq_m)
        g.set_codebooks(dev(cb))
        o.set_codebooks(cb)
    g.add(dev(w.base))
    o.add(w.base)
    torch.cuda.synchronize()
    return g, o


@pytest.mark.parametrize("pq_m", [0, 16])
def test_requests_larger_than_their_slice_use_the_reserve(pq_m):
    """A slice holds 64 x 200 entries; a batch of 64 queries has about 64 x 3,750
    candidates.  The first few queries fit, the others get room in the chunk the
    request leases."""
    w = small_set()
    print(f"[case] overflow reserve, workload={w.name} pq_m={pq_m}", flush=True)
    g, o = build(w, candidates_per_query=200, overflow_candidates=400_000, pq_m=pq_m)
    st = g.pool_stats()
    assert st.overflow_chunks == 4 and st.overflow_chunk_entries >= 400_000 and st.overflow_chunks_leased == 0
    for b in range(3):  # the same resource and the same reserve again and again
        q = w.queries[b * 64:(b + 1) * 64]
        d, i = g.search(dev(q), w.k, w.nprobe)
        torch.cuda.synchronize()
        assert g.poll_error() == 0
        rd, ri = o.search(q, w.k, w.nprobe)
        assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6)
        st = g.pool_stats()
        assert st.overflow_chunks_leased == 0, "the chunk was not returned"
    g.close()


def test_without_a_reserve_the_request_reports_escratch():
    w = small_set()
    print(f"[case] no reserve, workload={w.name}", flush=True)
    g, o = build(w, candidates_per_query=200, overflow_candidates=0)
    assert g.pool_stats().overflow_chunks == 0
    q = w.queries[:64]
    d, i = g.search(dev(q), w.k, w.nprobe)
    torch.cuda.synchronize()
    assert g.poll_error() == rtams.ESCRATCH
    # the queries that did fit are answered in full, the others come back empty
    rd, ri = o.search(q, w.k, w.nprobe)
    i = i.cpu().numpy()
    answered = (i >= 0).all(axis=1)
    assert 0 < answered.sum() < 64 and (i[~answered] == -1).all()
    assert_topk_matches(w.metric, d.cpu().numpy()[answered], i[answered], rd[answered], ri[answered], rtol=RTOL,
                        atol=1e-6)
    # A search that ran out of scratch is no reason to refuse vectors: the insert stream goes on, the
    # new vectors are there, smaller searches are answered; the flag stays until it is cleared.
    g.add(dev(w.inserts)); o.add(w.inserts)
    torch.cuda.synchronize()
    g.validate()
    assert np.array_equal(g.list_sizes(), o.list_sizes()) and g.pool_stats().ntotal == o.ntotal
    q = w.queries[64:66]
    d, i = g.search(dev(q), w.k, w.nprobe)
    torch.cuda.synchronize()
    rd, ri = o.search(q, w.k, w.nprobe)
    assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6)
    assert g.poll_error() == rtams.ESCRATCH
    g.clear_error()
    assert g.poll_error() == 0
    g.close()


def test_a_reserve_that_is_too_small_serves_whom_it_can_and_is_given_back():
    w = small_set()
    print(f"[case] small reserve, workload={w.name}", flush=True)
    g, o = build(w, candidates_per_query=200, overflow_candidates=40_000)
    q = w.queries[:64]
    d, i = g.search(dev(q), w.k, w.nprobe)
    torch.cuda.synchronize()
    assert g.poll_error() == rtams.ESCRATCH
    rd, ri = o.search(q, w.k, w.nprobe)
    i = i.cpu().numpy()
    answered = (i >= 0).all(axis=1)
    assert 5 < answered.sum() < 64
    assert_topk_matches(w.metric, d.cpu().numpy()[answered], i[answered], rd[answered], ri[answered], rtol=RTOL,
                        atol=1e-6)
    assert g.pool_stats().overflow_chunks_leased == 0
    g.close()


def test_concurrent_requests_share_the_reserve():
    """Four host threads, each with its own stream, search at once; every request
    overflows its slice and leases one of the four chunks.  Results are the
    oracle's, and in the end every chunk is back."""
    w = small_set()
    print(f"[case] shared reserve under 4 streams, workload={w.name}", flush=True)
    g, o = build(w, candidates_per_query=200, overflow_candidates=64 * 4_500, n_resources=4)
    rd, ri = o.search(w.queries, w.k, w.nprobe)
    qd = dev(w.queries)
    errors, results = [], {}

    def worker(t):
        try:
            s = torch.cuda.Stream()
            for rep in range(6):
                b = (t + 4 * rep) % 8
                od = torch.empty((64, w.k), dtype=torch.float32, device="cuda:0")
                oi = torch.empty((64, w.k), dtype=torch.int64, device="cuda:0")
                while True:
                    try:
                        g.search(qd[b * 64:(b + 1) * 64], w.k, w.nprobe, od, oi, stream=s)
                        break
                    except rtams.RtamsError as e:
                        if e.code != rtams.EBUSY:
                            raise
                s.synchronize()
                results[(t, rep)] = (b, od.cpu().numpy(), oi.cpu().numpy())
        except Exception as e:  # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    assert g.poll_error() == 0
    for (t, rep), (b, d, i) in results.items():
        assert_topk_matches(w.metric, d, i, rd[b * 64:(b + 1) * 64], ri[b * 64:(b + 1) * 64], rtol=RTOL, atol=1e-6,
                            what=f"thread {t} request {rep}")
    assert g.pool_stats().overflow_chunks_leased == 0
    g.close()


def test_more_requests_in_need_than_chunks():
    """One chunk, four streams: at any time at most one request holds it; the
    queries of the others that do not fit their slice come back empty (ESCRATCH),
    nothing is corrupted, and whatever is answered is right."""
    w = small_set()
    print(f"[case] one chunk under 4 streams, workload={w.name}", flush=True)
    g, o = build(w, candidates_per_query=200, overflow_candidates=64 * 4_500, n_resources=4, overflow_chunks=1)
    rd, ri = o.search(w.queries, w.k, w.nprobe)
    qd = dev(w.queries)
    errors, results = [], {}

    def worker(t):
        try:
            s = torch.cuda.Stream()
            for rep in range(6):
                b = (t + 4 * rep) % 8
                od = torch.empty((64, w.k), dtype=torch.float32, device="cuda:0")
                oi = torch.empty((64, w.k), dtype=torch.int64, device="cuda:0")
                while True:
                    try:
                        g.search(qd[b * 64:(b + 1) * 64], w.k, w.nprobe, od, oi, stream=s)
                        break
                    except rtams.RtamsError as e:
                        if e.code != rtams.EBUSY:
                            raise
                s.synchronize()
                results[(t, rep)] = (b, od.cpu().numpy(), oi.cpu().numpy())
        except Exception as e:  # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    full = 0
    for (t, rep), (b, d, i) in results.items():
        answered = (i >= 0).all(axis=1)
        assert (i[~answered] == -1).all() and answered.sum() >= 2
        full += int(answered.all())
        sl = slice(b * 64, (b + 1) * 64)
        assert_topk_matches(w.metric, d[answered], i[answered], rd[sl][answered], ri[sl][answered], rtol=RTOL,
                            atol=1e-6, what=f"thread {t} request {rep}")
    assert full >= 1 and g.pool_stats().overflow_chunks_leased == 0
    g.close()
