"""In-place rearrangement on the GPU: the invariants the paper's Rearrangement
algorithm must keep (logical content of every list, blocks in use, fewer header
jumps), the Exceed() trigger, and searches running while blocks move."""
import threading

import numpy as np
import pytest
import torch

from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import assert_lists_equal, dev, make_pair
from tests.helpers import assert_topk_matches

pytestmark = pytest.mark.gpu


def interleaved(nlist=3, d=8, T=64, rounds=6, seed=3, threshold=0, pool_blocks=200, settle=False):
    """Lists grown in turn, one block at a time, so every chain is scattered.  settle: wait for every
    batch, so that what it made exceed is known to the next add (which then carries the round)."""
    rng = np.random.default_rng(seed)
    C = (np.eye(nlist, d) * 10).astype(np.float32)
    w = synth.Workload("interleaved", "l2", d, nlist, T, nlist, 10, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, seed)
    g, o = make_pair(w, pool_blocks=pool_blocks, rearrange_threshold=threshold, candidates_per_query=8192)
    for r in range(rounds):
        for k in range(nlist):
            y = (C[k] + 0.5 * rng.standard_normal((T, d))).astype(np.float32)
            g.add(dev(y)); o.add(y)
            if settle:
                torch.cuda.synchronize()
    return w, g, o, rng


def open_one_more_block_each(w, g, o, rng):
    """One vector into every list, each opening a new block.  (Near a full pool add() refuses what MAY
    need more blocks than are left: a batch of one vector can need only one.)"""
    for k in range(w.nlist):
        y = (w.centroids[k:k + 1] + 0.5 * rng.standard_normal((1, w.d))).astype(np.float32)
        g.add(dev(y)); o.add(y)
        torch.cuda.synchronize()


def runs_of(g, k):
    return g.list_info(k)[1]


def test_rearrange_makes_a_chain_contiguous_and_keeps_every_list():
    w, g, o, _ = interleaved()
    g.validate()
    before = g.pool_stats().blocks_in_use
    chains = [g.list_chain(k) for k in range(3)]
    assert all(len(c) == 6 for c in chains) and runs_of(g, 0) == 6   # one jump per block
    g.rearrange(0)
    g.validate()
    c0 = g.list_chain(0)
    assert runs_of(g, 0) == 1 and np.array_equal(c0, c0[0] + np.arange(6))
    assert g.pool_stats().blocks_in_use == before
    assert_lists_equal(g, o)                                  # victims and target keep their content
    for k in (1, 2):                                          # victims can be compacted afterwards
        g.rearrange(k)
        g.validate()
        assert runs_of(g, k) == 1
    assert g.pool_stats().blocks_in_use == before
    assert_lists_equal(g, o)
    g.add(dev(w.centroids)); o.add(w.centroids)               # the index keeps working
    g.validate()
    assert_lists_equal(g, o)
    g.close()


def test_rearrange_into_free_fresh_and_own_blocks():
    """Targets that were never handed out, targets on the free stack, and targets
    held by a later block of the same chain."""
    w, g, o, rng = interleaved(nlist=2, rounds=4, pool_blocks=64)
    g.rearrange(1)                       # list 1 starts at block 1: its last target is past cur_P
    g.validate()
    assert runs_of(g, 1) == 1
    g.rearrange(0)                       # list 0 now finds free-stack blocks at its targets
    g.validate()
    assert runs_of(g, 0) == 1
    st = g.pool_stats()
    assert st.blocks_in_use == 8 and st.blocks_free + st.blocks_in_use == st.blocks_handed_out
    assert_lists_equal(g, o)
    for r in range(3):                   # grow both again, then compact the one that got scattered
        for k in (1, 0):
            y = (w.centroids[k] + 0.5 * rng.standard_normal((64, w.d))).astype(np.float32)
            g.add(dev(y)); o.add(y)
    g.rearrange(0); g.rearrange(1); g.rearrange(0)
    g.validate()
    assert runs_of(g, 0) == 1
    assert_lists_equal(g, o)
    g.close()


def test_rearrangement_with_a_single_spare_block_compacts_the_chain_round_by_round():
    """Moving the occupants of the target range out needs one spare block each for a while.  A pool
    with ONE free block (the paper's one temporary segment) still gets there: every round moves what
    the spare blocks allow, and the call goes on until the chain is contiguous.  Lists equal the
    oracle's throughout, blocks in use never change."""
    print("[case] rearrangement with one spare block", flush=True)
    w, g, o, rng = interleaved(nlist=2, rounds=5, pool_blocks=13)
    open_one_more_block_each(w, g, o, rng)                             # 12 blocks in use, 1 spare
    assert g.list_chain(0).tolist() == [0, 2, 4, 6, 8, 10] and g.list_chain(1).tolist() == [1, 3, 5, 7, 9, 11]
    for k in (1, 0):
        g.rearrange(k)                                                 # 5 occupants in the way, 1 spare block
        g.validate()
        assert g.poll_error() == 0
        c = g.list_chain(k)
        assert runs_of(g, k) == 1 and np.array_equal(c, c[0] + np.arange(6))
        st = g.pool_stats()
        assert st.blocks_in_use == 12 and st.rearrangement_state == 0
        assert_lists_equal(g, o)
    y = (w.centroids[:1] + 0.5 * rng.standard_normal((1, w.d))).astype(np.float32)
    g.add(dev(y)); o.add(y)                                            # the index keeps working
    g.validate()
    assert_lists_equal(g, o)
    g.close()


def test_rearrangement_in_a_full_pool_reports_that_it_is_stalled():
    """No spare block at all: nothing can move.  The call says so (ENOSPARE), every chain is as it was,
    Exceed() keeps holding for the list, and searches and the index go on as usual."""
    print("[case] rearrangement in a full pool", flush=True)
    w, g, o, rng = interleaved(nlist=2, rounds=5, pool_blocks=12, threshold=10_000)
    open_one_more_block_each(w, g, o, rng)                             # 12 blocks in use, none spare
    assert g.pool_stats().blocks_in_use == 12
    chains = [g.list_chain(k).copy() for k in range(2)]
    for k in (1, 0):
        with pytest.raises(rtams.RtamsError) as e:
            g.rearrange(k)
        assert e.value.code == rtams.ENOSPARE
        g.validate()
        assert g.poll_error() == 0
        assert [g.list_chain(j).tolist() for j in range(2)] == [c.tolist() for c in chains]
        assert g.pool_stats().rearrangement_state == 2
    assert_lists_equal(g, o)
    q = (w.centroids + 0.1).astype(np.float32)
    dd, ii = g.search(dev(q), 10, 2)
    rd, ri = o.search(q, 10, 2)
    assert_topk_matches("l2", dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=1e-4, atol=1e-6)
    g.close()


def test_exceeding_lists_in_a_nearly_full_pool_are_compacted_a_few_blocks_at_a_time():
    """Exceed() armed while the pool fills up to its last block: the rounds the adds carry move what the
    spare blocks of the moment allow and keep the flag until the chain is contiguous; in the end either
    nothing exceeds, or the pool is full and rearrange(-1) says that it is stalled without clearing
    anything."""
    w, g, o, rng = interleaved(nlist=2, rounds=5, pool_blocks=12, threshold=150, settle=True)
    open_one_more_block_each(w, g, o, rng)
    g.validate()
    assert_lists_equal(g, o)
    st = g.pool_stats()
    assert st.blocks_in_use == 12
    if st.lists_exceeding:
        with pytest.raises(rtams.RtamsError) as e:
            g.rearrange(-1)
        assert e.value.code == rtams.ENOSPARE
        assert g.pool_stats().lists_exceeding == st.lists_exceeding
        g.validate()
        assert_lists_equal(g, o)
    g.close()


def test_the_last_batch_exceeds_and_nothing_follows():
    """An add only carries the round that an EARLIER batch made necessary.  After the last batch of a
    burst the list stays flagged (and scattered) until the caller asks: rearrange(-1) then compacts it."""
    w, g, o, rng = interleaved(nlist=3, rounds=3, threshold=250)       # 192 per list: no trigger
    y = (w.centroids[2] + 0.5 * rng.standard_normal((64, w.d))).astype(np.float32)  # 256 > 250
    g.add(dev(y)); o.add(y)
    st = g.pool_stats()
    assert st.lists_exceeding == 1 and runs_of(g, 2) == 3              # blocks 2 | 5 | 8 9: nothing has moved yet
    g.rearrange(-1)
    g.validate()
    st = g.pool_stats()
    assert st.lists_exceeding == 0 and st.rearrangement_state == 0 and runs_of(g, 2) == 1
    assert g.list_info(2)[2] == 0
    assert_lists_equal(g, o)
    g.close()


def test_exceed_triggers_rearrangement_behind_the_batch():
    """Exceed() is evaluated when a batch is published; the round is enqueued by
    the next add (or by rearrange(-1)).  The oracle rearranges at once; the logical
    content must agree at every point, the block structure must stay valid."""
    w, g, o, rng = interleaved(nlist=3, rounds=2, threshold=200)   # 128 per list so far: no trigger
    assert g.pool_stats().lists_exceeding == 0 and o.n_rearrange == 0
    y = (w.centroids[1] + 0.5 * rng.standard_normal((73, w.d))).astype(np.float32)   # 201 > 200
    g.add(dev(y)); o.add(y)
    assert g.pool_stats().lists_exceeding == 1 and o.n_rearrange == 1
    assert runs_of(g, 1) == 3                                      # blocks 1 | 4 | 6 7
    g.add(dev(w.centroids[:1])); o.add(w.centroids[:1])            # carries the round
    g.validate()
    assert g.pool_stats().lists_exceeding == 0 and runs_of(g, 1) == 1
    assert g.list_info(1)[2] == 0                                  # counter restarts
    assert_lists_equal(g, o)
    y = (w.centroids[2] + 0.5 * rng.standard_normal((72, w.d))).astype(np.float32)   # exactly 200: no trigger
    g.add(dev(y)); o.add(y)
    assert g.pool_stats().lists_exceeding == 0 and o.n_rearrange == 1
    g.close()


def test_searches_stay_correct_while_blocks_move():
    w = synth.skewed_l2("zipf-rearr", 41, d=32, n_base=40_000, nlist=32, block_vecs=64, n_queries=256,
                        n_inserts=64, nprobe=8, k=20)
    g, o = make_pair(w, pool_blocks=1400, n_resources=8)
    for b in range(0, len(w.base), 500):                   # many small batches: scattered chains
        g.add(dev(w.base[b:b + 500])); o.add(w.base[b:b + 500])
    torch.cuda.synchronize()
    q = dev(w.queries)
    rd, ri = o.search(w.queries, w.k, w.nprobe)
    stop, bad, done = threading.Event(), [], [0]
    streams = [torch.cuda.Stream() for _ in range(3)]

    def searcher(s):
        od = torch.empty((256, w.k), dtype=torch.float32, device="cuda:0")
        oi = torch.empty((256, w.k), dtype=torch.int64, device="cuda:0")
        while not stop.is_set():
            try:
                g.search(q, w.k, w.nprobe, od, oi, stream=s)
            except rtams.RtamsError as e:
                if e.code == rtams.EBUSY:
                    s.synchronize()
                    continue
                bad.append(str(e)); return
            s.synchronize()
            try:
                assert_topk_matches("l2", od.cpu().numpy(), oi.cpu().numpy(), rd, ri, rtol=1e-4, atol=1e-6)
            except AssertionError as e:
                bad.append(str(e)); return
            done[0] += 1

    threads = [threading.Thread(target=searcher, args=(s,)) for s in streams]
    for t in threads:
        t.start()
    data = torch.cuda.Stream()
    order = np.argsort(-g.list_sizes())
    for rep in range(3):                                   # compacting one list scatters its neighbours
        for k in order[:12]:
            g.rearrange(int(k), stream=data)
        data.synchronize()
    stop.set()
    for t in threads:
        t.join()
    assert not bad, bad[0]
    assert done[0] > 0
    g.validate()
    assert_lists_equal(g, o)
    g.close()


def test_rearrange_all_handles_every_exceeding_list():
    """Several lists pass T_m' in ONE batch; rearrange(-1) must bring all of them in order (one round
    handles one list), not just the first."""
    w, g, o, rng = interleaved(nlist=4, rounds=3, threshold=250)     # 192 per list, scattered: nobody exceeds
    assert g.pool_stats().lists_exceeding == 0
    y = np.concatenate([(w.centroids[k] + 0.5 * rng.standard_normal((70, w.d))).astype(np.float32)
                        for k in (0, 2, 3)])                         # 262 > 250 for three lists at once
    perm = rng.permutation(len(y))
    g.add(dev(y[perm])); o.add(y[perm])
    assert g.pool_stats().lists_exceeding == 3
    g.rearrange(-1)
    g.validate()
    assert g.pool_stats().lists_exceeding == 0
    for k in (0, 2, 3):
        assert g.list_info(k)[2] == 0                                # every one of them had its round
    assert runs_of(g, 3) == 1    # the last one handled is in one run (an earlier one may have given way to a later)
    assert_lists_equal(g, o)
    g.close()
