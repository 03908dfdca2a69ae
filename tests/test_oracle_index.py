"""Pins of the oracle's insertion, block model and rearrangement: invariants
recomputed independently, closed forms from the Insertion algorithm, and the
numbers and the scenario the paper itself gives."""
import os

import numpy as np
import pytest

from oracle.oracle import EPOOL, OracleError, OracleIndex
from paper_2408_02937_amd import synth
from tests.helpers import brute_force_scores, order_by_score_then_id

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        out[key] = [int(v) for v in vals]
    return out


def test_every_id_once_in_the_list_of_its_nearest_centroid():
    w = synth.config(1)
    ix = OracleIndex(w.d, w.nlist, "l2", w.block_vecs)
    ix.set_centroids(w.centroids)
    ix.add(w.base)
    for b in range(0, len(w.inserts), w.insert_batch):
        ix.add(w.inserts[b:b + w.insert_batch])                 # ids default to ntotal + i
    allv = np.concatenate([w.base, w.inserts])
    n = len(allv)
    assert ix.ntotal == n and ix.list_sizes().sum() == n       # gid = sum of list lengths
    seen = np.zeros(n, dtype=np.int64)
    where = np.full(n, -1)
    for k in range(w.nlist):
        ids, x = ix.list_export(k)
        np.add.at(seen, ids, 1)
        where[ids] = k
        assert np.array_equal(x, allv[ids])                     # vector bits travel with the id
        assert np.all(np.diff(ids) > 0)                         # sequential insertion order
    assert np.all(seen == 1)
    for r in range(0, n, 7):                                    # independent nearest centroid
        s = brute_force_scores("l2", w.centroids, allv[r])
        assert where[r] == order_by_score_then_id("l2", s, np.arange(w.nlist))[0]
    assert np.array_equal(ix.assign(allv[:500]), where[:500])


def test_assignment_metric_and_tie_break():
    C = np.array([[1, 0], [1, 0], [0, 2], [0, -1]], dtype=np.float32)
    y = np.array([[0.9, 0.1], [0.1, 0.6], [0, -5]], dtype=np.float32)
    l2 = OracleIndex(2, 4, "l2", 2); l2.set_centroids(C)
    ip = OracleIndex(2, 4, "ip", 2); ip.set_centroids(C)
    assert l2.assign(y).tolist() == [0, 0, 3]                  # equal centroids 0/1: lowest index
    assert ip.assign(y).tolist() == [0, 2, 3]                  # largest inner product


@pytest.mark.parametrize("T_m", [1, 3, 64])
def test_block_closed_forms(T_m):
    """did -> (mid, moff) = (did / T_m, did % T_m); a list of n vectors owns
    ceil(n / T_m) blocks; blocks in use = cur_P - free."""
    rng = np.random.default_rng(T_m)
    d, nlist = 4, 5
    C = rng.standard_normal((nlist, d), dtype=np.float32)
    ix = OracleIndex(d, nlist, "l2", T_m, pool_blocks=10_000)
    ix.set_centroids(C)
    total_blocks = 0
    for batch in range(6):
        ix.add(rng.standard_normal((37, d), dtype=np.float32))
        sizes = ix.list_sizes()
        nb = [(int(s) + T_m - 1) // T_m for s in sizes]
        assert [ix.list_blocks(k) for k in range(nlist)] == nb
        assert ix.blocks_in_use == sum(nb) == ix.cur_P - ix.nfree
        total_blocks = sum(nb)
    chains = [ix.list_chain(k) for k in range(nlist)]
    allb = np.concatenate(chains)
    assert len(set(allb.tolist())) == total_blocks             # no block owned twice
    for k in range(nlist):
        for did in range(ix.list_size(k)):
            assert ix.slot(k, did) == (chains[k][did // T_m], did % T_m)


def test_pad_memory_figure_of_the_paper():
    g = read_golden("pad_memory.txt")
    nlist, T_m, d = g["nlist"][0], g["block_vecs"][0], g["d"][0]
    rng = np.random.default_rng(0)
    C = rng.standard_normal((nlist, d), dtype=np.float32)
    ix = OracleIndex(d, nlist, "l2", T_m, pool_blocks=nlist)
    ix.set_centroids(C)
    ix.add(C)                                                   # one vector per list
    assert np.all(ix.list_sizes() == 1) and ix.blocks_in_use == nlist
    vec_bytes = ix.blocks_in_use * T_m * d * 4
    assert g["min_bytes"][0] <= vec_bytes <= g["max_bytes"][0]
    assert ix.pool_bytes_in_use(0) == nlist * T_m * (8 + 4 * d)


def test_pool_exhaustion_leaves_no_trace():
    C = np.eye(2, dtype=np.float32)
    ix = OracleIndex(2, 2, "ip", 2, pool_blocks=3)
    ix.set_centroids(C)
    ix.add(np.array([[1, 0]] * 4, dtype=np.float32))           # 2 blocks of list 0
    with pytest.raises(OracleError) as e:
        ix.add(np.array([[0, 1]] * 3, dtype=np.float32))       # would need 2 more
    assert e.value.code == EPOOL
    assert ix.ntotal == 4 and ix.blocks_in_use == 2 and ix.list_size(1) == 0
    ix.add(np.array([[0, 1]] * 2, dtype=np.float32))           # exactly fits
    assert ix.blocks_in_use == 3


def two_list_index(T_m, T_mp, alloc, pool_blocks=64):
    """Two lists A=0, B=1 in 2-d; one block is opened per entry of alloc."""
    C = np.array([[1, 0], [0, 1]], dtype=np.float32)
    ix = OracleIndex(2, 2, "ip", T_m, rearrange_threshold=T_mp, pool_blocks=pool_blocks)
    ix.set_centroids(C)
    for who in alloc:                                           # fill one whole block each time
        ix.add(np.repeat(C[who:who + 1], T_m, axis=0) * np.float32(1 + ix.ntotal))
    return ix


def test_figure1_rearrangement_scenario():
    g = read_golden("figure1_chain.txt")
    ix = two_list_index(2, 0, g["alloc"])
    assert ix.list_chain(0).tolist() == g["chain_A_before"]
    assert ix.list_chain(1).tolist() == g["chain_B_before"]
    assert ix.list_jumps(0) == g["jumps_A_before"][0]
    before = [ix.list_export(k) for k in range(2)]
    in_use = ix.blocks_in_use
    ix.rearrange(0)
    assert ix.list_chain(0).tolist() == g["chain_A_after"]
    assert ix.list_chain(1).tolist() == g["chain_B_after"]
    assert ix.list_jumps(0) == g["jumps_A_after"][0]
    for k in range(2):                                          # logical content untouched
        ids, x = ix.list_export(k)
        assert np.array_equal(ids, before[k][0]) and np.array_equal(x, before[k][1])
    assert ix.blocks_in_use == in_use
    ix.rearrange(1)                                             # the victim can be re-compacted
    assert ix.list_jumps(1) == 0 and ix.blocks_in_use == in_use
    owned = np.concatenate([ix.list_chain(0), ix.list_chain(1)])
    assert len(set(owned.tolist())) == len(owned)


def test_rearrangement_into_free_and_fresh_blocks():
    """The neighbour may also be a returned block or one never handed out."""
    ix = two_list_index(2, 0, [0, 1, 0, 1, 0])                  # A = 0 2 4, B = 1 3
    ix.rearrange(0)                                             # A = 0 1 2, B = 4 3
    assert ix.list_chain(0).tolist() == [0, 1, 2] and ix.list_chain(1).tolist() == [4, 3]
    ix.rearrange(1)                                             # B wants 4 5: 5 is fresh, 3 is freed
    assert ix.list_chain(1).tolist() == [4, 5] and ix.cur_P == 6 and ix.nfree == 1
    assert ix.blocks_in_use == 5
    ix.add(np.array([[1, 0]] * 2, dtype=np.float32))            # next block comes off the free stack
    assert ix.list_chain(0).tolist() == [0, 1, 2, 3] and ix.nfree == 0


def test_a_rearranged_list_can_be_the_next_victim():
    """Worked by hand from the Rearrangement algorithm (exchange of the two blocks'
    contents and owners): B = 0 2 4, A = 1 3.  Compacting A exchanges 3 with 2
    (A = 1 2, B = 0 3 4).  Compacting B then takes both of A's blocks, the one A
    was opened with and the one it was just given: 1 against 3, then 2 against
    4 (B = 0 1 2, A = 3 4).  Every block stays in exactly one chain."""
    ix = two_list_index(2, 0, [1, 0, 1, 0, 1])
    assert ix.list_chain(1).tolist() == [0, 2, 4] and ix.list_chain(0).tolist() == [1, 3]
    before = [ix.list_export(k) for k in range(2)]
    ix.rearrange(0)
    assert ix.list_chain(0).tolist() == [1, 2] and ix.list_chain(1).tolist() == [0, 3, 4]
    ix.rearrange(1)
    assert ix.list_chain(1).tolist() == [0, 1, 2] and ix.list_chain(0).tolist() == [3, 4]
    assert ix.list_jumps(0) == 0 and ix.list_jumps(1) == 0 and ix.blocks_in_use == 5 and ix.nfree == 0
    for k in range(2):
        ids, x = ix.list_export(k)
        assert np.array_equal(ids, before[k][0]) and np.array_equal(x, before[k][1])
    assert [ix.slot(0, did) for did in range(4)] == [(3, 0), (3, 1), (4, 0), (4, 1)]


def test_rearrangement_onto_a_block_of_the_free_stack_in_a_full_pool():
    """Worked by hand, pool of exactly 8 blocks.  A = 0 2 5, B = 1 3 4.  Compacting
    A exchanges 1 and 2 with B's first block in turn (A = 0 1 2, B = 5 3 4).  B now
    starts at the frontier: its targets 6 and 7 were never handed out, its blocks 3
    and 4 go to the free stack (4 on top) and the pool's bump pointer is at its
    end.  A's next block comes off the stack (4: the pool is full otherwise, the
    add must not be refused); compacting A then finds its target 3 ON the stack:
    3 leaves the stack, 4 returns to it.  Later blocks: 4 again, then nothing."""
    from oracle.oracle import OracleError
    ix = two_list_index(2, 0, [0, 1, 0, 1, 1, 0], pool_blocks=8)
    C = np.array([[1, 0], [0, 1]], dtype=np.float32)
    block_for = lambda who: np.repeat(C[who:who + 1], 2, axis=0)
    assert ix.list_chain(0).tolist() == [0, 2, 5] and ix.list_chain(1).tolist() == [1, 3, 4]
    ix.rearrange(0)
    assert ix.list_chain(0).tolist() == [0, 1, 2] and ix.list_chain(1).tolist() == [5, 3, 4]
    ix.rearrange(1)
    assert ix.list_chain(1).tolist() == [5, 6, 7] and ix.cur_P == 8 and ix.nfree == 2 and ix.blocks_in_use == 6
    ix.add(block_for(0))                                        # bump pointer exhausted, two blocks on the stack
    assert ix.list_chain(0).tolist() == [0, 1, 2, 4] and ix.nfree == 1
    ix.rearrange(0)
    assert ix.list_chain(0).tolist() == [0, 1, 2, 3] and ix.nfree == 1 and ix.blocks_in_use == 7
    ix.add(block_for(1))
    assert ix.list_chain(1).tolist() == [5, 6, 7, 4] and ix.nfree == 0 and ix.blocks_in_use == 8
    with pytest.raises(OracleError):
        ix.add(block_for(0))                                    # now the pool is full
    owned = np.concatenate([ix.list_chain(0), ix.list_chain(1)])
    assert sorted(owned.tolist()) == list(range(8))


def test_rearrangement_stops_at_the_end_of_the_pool():
    """The same start in a pool of 7 blocks: B's second target (7) does not
    exist, the list stays compacted as far as the pool reaches."""
    ix = two_list_index(2, 0, [0, 1, 0, 1, 1, 0], pool_blocks=7)
    ix.rearrange(0)
    before = ix.list_export(1)
    ix.rearrange(1)
    assert ix.list_chain(1).tolist() == [5, 6, 4] and ix.cur_P == 7 and ix.nfree == 1 and ix.blocks_in_use == 6
    assert ix.list_jumps(1) == 1
    ids, x = ix.list_export(1)
    assert np.array_equal(ids, before[0]) and np.array_equal(x, before[1])


def test_exceed_is_a_strict_inequality():
    T_m, T_mp = 2, 6
    C = np.array([[1, 0], [0, 1]], dtype=np.float32)
    ix = OracleIndex(2, 2, "ip", T_m, rearrange_threshold=T_mp, pool_blocks=64)
    ix.set_centroids(C)
    a, b = C[0:1], C[1:2]
    for _ in range(3):                                          # interleave so A's chain is scattered
        ix.add(np.repeat(a, 2, axis=0)); ix.add(np.repeat(b, 2, axis=0))
    assert ix.list_online(0) == T_mp and ix.n_rearrange == 0    # exactly T_m' does not trigger
    assert ix.list_jumps(0) == 2
    ix.add(a)                                                   # T_m' + 1 does
    assert ix.n_rearrange == 1 and ix.list_online(0) == 0 and ix.list_jumps(0) == 0
    assert ix.list_size(0) == 7 and ix.list_blocks(0) == 4
