"""Helpers of the GPU parity tests: build the HIP index and the oracle from the
same workload, compare list contents canonically."""
from __future__ import annotations

import threading

import numpy as np
import torch

from oracle.oracle import OracleIndex
from paper_2408_02937_amd import rtams
from tests.helpers import ATOL, RTOL, assert_topk_matches


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def scan_modes(g, modes=(2, 0)):
    """Runs the body of a for loop once per arithmetic of the list scan: dot products on the matrix
    cores whatever the batch size (2; by default, 1, flat float lists take them from 64 queries on),
    then on the vector unit (0).  Answers must agree with the oracle either way.  The default is
    restored afterwards."""
    try:
        for m in modes:
            g.set_param("scan_mfma", m)
            yield m
    finally:
        g.set_param("scan_mfma", 1)


def make_pair(w, pool_blocks=None, rearrange_threshold=0, max_batch=256, max_k=128, max_nprobe=64,
              candidates_per_query=None, n_resources=4, max_add_batch=65536, storage="f32"):
    """(gpu index, oracle index) over workload w, centroids set, nothing added."""
    n_all = len(w.base) + len(w.inserts)
    if pool_blocks is None:
        pool_blocks = n_all // w.block_vecs + 2 * w.nlist + 8
    if candidates_per_query is None:
        candidates_per_query = n_all + 64
    g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=pool_blocks,
                    rearrange_threshold=rearrange_threshold, n_resources=n_resources,
                    max_batch=max_batch, max_k=max_k, max_nprobe=min(max_nprobe, w.nlist),
                    max_add_batch=max_add_batch, candidates_per_query=candidates_per_query, storage=storage)
    g.set_centroids(dev(w.centroids))
    o = OracleIndex(w.d, w.nlist, w.metric, w.block_vecs, rearrange_threshold=rearrange_threshold,
                    pool_blocks=pool_blocks)
    o.set_centroids(w.centroids)
    if storage != "f32":
        o.set_storage(storage)
    return g, o


def assert_lists_equal(g, o, batch_bounds=None):
    """Bit-exact list contents as sets of (id -> vector bits); block arithmetic;
    and, inside every list, all entries of batch b before those of batch b+1."""
    sizes = g.list_sizes()
    assert np.array_equal(sizes, o.list_sizes()), "list lengths differ"
    T = g.block_vecs
    for k in range(g.nlist):
        gi, gx = g.list_export(k)
        gi, gx = gi.cpu().numpy(), gx.cpu().numpy()
        oi, ox = o.list_export(k)
        og, oo = np.argsort(gi, kind="stable"), np.argsort(oi, kind="stable")
        assert np.array_equal(gi[og], oi[oo]), f"list {k}: ids differ"
        assert np.array_equal(gx[og].view(np.uint32), ox[oo].view(np.uint32)), f"list {k}: vector bits differ"
        blocks, runs, online = g.list_info(k)
        assert blocks == (int(sizes[k]) + T - 1) // T == o.list_blocks(k)
        if batch_bounds is not None and len(gi):
            # ids were given as ntotal + i, so the batch of an entry follows from its id
            b = np.searchsorted(batch_bounds, gi, side="right")
            assert np.all(np.diff(b) >= 0), f"list {k}: batches interleave"
    st = g.pool_stats()
    assert st.ntotal == o.ntotal and st.blocks_in_use == o.blocks_in_use


def _matches(metric, d, i, rd, ri, atol=ATOL):
    try:
        assert_topk_matches(metric, d[None], i[None], rd[None], ri[None], rtol=RTOL, atol=atol)
        return True
    except AssertionError:
        return False


def whole_batches_check(w, g, o, n_search_threads, atol=ATOL):
    """Base set in, then the insert stream batch by batch on a data stream while searcher threads
    query on streams of their own.  A search must see whole batches only: its answer equals the
    oracle's on SOME prefix of the batches, between those finished before it was submitted and those
    submitted before it finished; at rest the answers are exactly the oracle's on everything."""
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
    bad, checked = [], [0]

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
                ok = [p for p in range(lo, hi + 1)
                      if _matches(w.metric, d[r], i[r], expected[p][0][r], expected[p][1][r], atol)]
                if not ok:
                    bad.append(f"query {r}: no batch prefix in [{lo}, {hi}] explains the result"); return
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
    d, i = g.search(q, w.k, w.nprobe)                   # at rest: exactly the last prefix
    assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), expected[-1][0], expected[-1][1],
                        rtol=RTOL, atol=atol)
