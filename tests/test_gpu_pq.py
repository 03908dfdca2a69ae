"""Product-quantised lists: HIP path against the CPU oracle through the C ABI.
Codes, ids, list lengths and block counts bit for bit; scores within the
tolerance of the flat path (the GPU adds the table entries in fp32, the oracle
in double); exact where the data make fp32 exact."""
import numpy as np
import pytest
import torch

from oracle.oracle import OracleIndex
from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import dev, whole_batches_check
from tests.helpers import assert_topk_matches, ATOL_PQ, RTOL

pytestmark = pytest.mark.gpu



def make_pq_pair(w, M, cb, pool_blocks=None, rearrange_threshold=0, n_resources=2, **kw):
    n_all = len(w.base) + len(w.inserts)
    if pool_blocks is None:
        pool_blocks = n_all // w.block_vecs + 2 * w.nlist + 8
    g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=pool_blocks,
                    rearrange_threshold=rearrange_threshold, n_resources=n_resources, max_batch=256, max_k=128,
                    max_nprobe=min(64, w.nlist), max_add_batch=65536, candidates_per_query=n_all + 64,
                    pq_m=M, **kw)
    g.set_centroids(dev(w.centroids))
    g.set_codebooks(dev(cb))
    o = OracleIndex(w.d, w.nlist, w.metric, w.block_vecs, rearrange_threshold=rearrange_threshold,
                    pool_blocks=pool_blocks)
    o.set_centroids(w.centroids)
    o.set_codebooks(cb)
    return g, o


def cases():
    return {
        # name: (workload, M)
        "byte-l2-m8": (synth.byte_valued_l2("pq-byte", 41, d=32, n_base=30_000, n_centres=40, nlist=64,
                                            block_vecs=128, n_queries=300, n_inserts=3_000, insert_batch=64,
                                            nprobe=8, k=100), 8),
        "unit-ip-m12": (synth.unit_ip("pq-ip", 42, d=96, n_base=40_000, n_centres=300, nlist=128,
                                      block_vecs=256, n_queries=300, n_inserts=2_048, insert_batch=512,
                                      nprobe=16, k=10), 12),
        "gauss-l2-m64": (synth.gaussian_l2("pq-gauss", 43, d=128, n_base=20_000, n_centres=100, nlist=50,
                                           block_vecs=64, n_queries=260, n_inserts=1_000, insert_batch=100,
                                           nprobe=10, k=50), 64),
    }


def assert_code_lists_equal(g, o):
    sizes = g.list_sizes()
    assert np.array_equal(sizes, o.list_sizes()), "list lengths differ"
    T = g.block_vecs
    for k in range(g.nlist):
        gi, gc = g.list_export_codes(k)
        gi, gc = gi.cpu().numpy(), gc.cpu().numpy()
        oi, oc = o.list_export_codes(k)
        a, b = np.argsort(gi, kind="stable"), np.argsort(oi, kind="stable")
        assert np.array_equal(gi[a], oi[b]), f"list {k}: ids differ"
        assert np.array_equal(gc[a], oc[b]), f"list {k}: codes differ"
        assert g.list_info(k)[0] == (int(sizes[k]) + T - 1) // T == o.list_blocks(k)
    st = g.pool_stats()
    assert st.ntotal == o.ntotal and st.blocks_in_use == o.blocks_in_use


@pytest.fixture(scope="module", params=list(cases().keys()))
def loaded(request):
    w, M = cases()[request.param]
    print(f"[case] pq workload={w.name} seed={w.seed} M={M}", flush=True)
    cb = synth.codebooks_from_rows(w.seed, w.base, M)
    g, o = make_pq_pair(w, M, cb)
    g.add(dev(w.base)); o.add(w.base)
    for b in range(0, len(w.inserts), w.insert_batch):
        chunk = w.inserts[b:b + w.insert_batch]
        g.add(dev(chunk)); o.add(chunk)
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    yield w, M, g, o
    g.close()


def test_codes_and_lists_are_bit_exact(loaded):
    w, M, g, o = loaded
    g.validate()
    assert_code_lists_equal(g, o)


@pytest.mark.parametrize("batch", [1, 7, 256])
def test_pq_search_matches_oracle(loaded, batch):
    w, M, g, o = loaded
    q = w.queries[:batch]
    d, i = g.search(dev(q), w.k, w.nprobe)
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    rd, ri = o.search(q, w.k, w.nprobe)
    assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd, ri, rtol=RTOL, atol=ATOL_PQ,
                        what=f"{w.name} batch {batch}")


def test_pq_search_all_lists_and_large_k(loaded):
    w, M, g, o = loaded
    nprobe = min(w.nlist, 64)
    q = w.queries[:32]
    d, i = g.search(dev(q), 128, nprobe)
    torch.cuda.synchronize()
    rd, ri = o.search(q, 128, nprobe)
    assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd, ri, rtol=RTOL, atol=ATOL_PQ)


def test_integer_valued_tables_make_the_scores_exact():
    """Byte-valued data and codebook entries: every table entry and every partial sum is an
    integer below 2^24, so ids (ties by id included) and scores must equal the oracle's."""
    w, M = cases()["byte-l2-m8"]
    cb = synth.codebooks_from_rows(w.seed, w.base, M)
    g, o = make_pq_pair(w, M, cb)
    base = np.concatenate([w.base, w.base[:500]])  # duplicates: exact ties (and many more from the coarse codes)
    g.add(dev(base)); o.add(base)
    for batch in (5, 256):
        q = w.queries[:batch]
        d, i = g.search(dev(q), w.k, w.nprobe)
        torch.cuda.synchronize()
        rd, ri = o.search(q, w.k, w.nprobe)
        assert np.array_equal(i.cpu().numpy(), ri)
        assert np.array_equal(d.cpu().numpy().astype(np.float64), rd)
    g.close()


@pytest.mark.parametrize("metric", ["l2", "ip"])
def test_lossless_quantiser_answers_like_the_flat_index(metric):
    """One dimension per sub-space, codebooks holding every byte value: the coded index must
    return what the oracle's FLAT index returns on byte-valued data."""
    rng = np.random.default_rng(5)
    d, nlist, n = 8, 6, 5000
    C = rng.integers(0, 256, (nlist, d)).astype(np.float32)
    x = rng.integers(0, 256, (n, d)).astype(np.float32)
    q = rng.integers(0, 256, (40, d)).astype(np.float32)
    cb = np.tile(np.arange(256, dtype=np.float32)[None, :, None], (d, 1, 1))
    w = synth.Workload("pq-lossless", metric, d, nlist, 64, 3, 20, x, C, q, np.zeros((0, d), np.float32), 1, 5)
    g, _ = make_pq_pair(w, d, cb)
    flat = OracleIndex(d, nlist, metric, 64, pool_blocks=4096)
    flat.set_centroids(C)
    g.add(dev(x)); flat.add(x)
    for k in range(nlist):
        gi, gc = g.list_export_codes(k)
        fi, fx = flat.list_export(k)
        a, b = np.argsort(gi.cpu().numpy(), kind="stable"), np.argsort(fi, kind="stable")
        assert np.array_equal(gc.cpu().numpy()[a], fx[b].astype(np.uint8))
    dd, ii = g.search(dev(q), 20, 3)
    fd, fi = flat.search(q, 20, 3)
    assert np.array_equal(ii.cpu().numpy(), fi)
    assert np.array_equal(dd.cpu().numpy().astype(np.float64), fd)
    g.close()


def test_rearrangement_moves_coded_blocks_intact():
    """Three lists filled in turn, so their chains interleave; rearranging makes each chain one
    run and changes neither a code nor an answer."""
    rng = np.random.default_rng(6)
    d, M, T = 16, 4, 64
    C = np.zeros((3, d), np.float32)
    C[1, 0], C[2, 0] = 100.0, 200.0
    x = (C[np.arange(6 * 3 * T) // T % 3] + rng.standard_normal((6 * 3 * T, d))).astype(np.float32)
    cb = synth.codebooks_from_rows(6, x, M)
    w = synth.Workload("pq-rearr", "l2", d, 3, T, 3, 10, x, C, x[:64], np.zeros((0, d), np.float32), T, 6)
    g, o = make_pq_pair(w, M, cb, pool_blocks=64)
    for b in range(0, len(x), T):
        g.add(dev(x[b:b + T])); o.add(x[b:b + T])
    g.validate()
    assert g.list_info(0)[1] == 6
    rd, ri = o.search(x[:64], 10, 3)
    for k in range(3):
        g.rearrange(k)
        g.validate()
        assert g.list_info(k)[1] == 1
        assert_code_lists_equal(g, o)
        dd, ii = g.search(dev(x[:64]), 10, 3)
        assert_topk_matches("l2", dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=RTOL, atol=ATOL_PQ)
    g.close()


def test_pq_state_and_argument_errors():
    C = np.zeros((4, 16), np.float32)
    for bad in (3, 68, 12):  # not a multiple of 4; above 64; does not divide d
        with pytest.raises(rtams.RtamsError):
            rtams.Index(16, 4, "l2", 64, pool_blocks=32, pq_m=bad)
    g = rtams.Index(16, 4, "l2", 64, pool_blocks=32, pq_m=4)
    g.set_centroids(dev(C))
    with pytest.raises(rtams.RtamsError):
        g.add(dev(np.ones((3, 16), np.float32)))          # no codebooks yet
    with pytest.raises(rtams.RtamsError):
        g.search(dev(np.ones((3, 16), np.float32)), 1, 1)
    g.set_codebooks(dev(np.zeros((4, 256, 4), np.float32)))
    g.add(dev(np.ones((3, 16), np.float32)))
    with pytest.raises(rtams.RtamsError):
        g.list_export(0)                                   # the lists hold codes, not vectors
    with pytest.raises(rtams.RtamsError):
        g.set_codebooks(dev(np.zeros((4, 256, 4), np.float32)))  # vectors are in
    ids, codes = g.list_export_codes(0)
    assert ids.cpu().numpy().tolist() == [0, 1, 2] and not codes.cpu().numpy().any()  # ties: lowest entry
    g.close()
    f = rtams.Index(16, 4, "l2", 64, pool_blocks=32)
    with pytest.raises((rtams.RtamsError, ValueError)):
        f.set_codebooks(dev(np.zeros((4, 256, 4), np.float32)))
    f.close()


def test_pq_search_sees_whole_batches_only():
    """Insertion into coded lists on the data stream while two threads search: every answer is the
    oracle's for some prefix of the batches (codes and ids of a batch become visible together)."""
    w = synth.gaussian_l2("pq-concurrent", 79, d=32, n_base=10_000, n_queries=64, n_inserts=2_000,
                          insert_batch=50, nlist=64, block_vecs=64)
    cb = synth.codebooks_from_rows(w.seed, w.base, 8)
    g, o = make_pq_pair(w, 8, cb, n_resources=8)
    whole_batches_check(w, g, o, 2, atol=ATOL_PQ)
    assert_code_lists_equal(g, o)
    g.close()


def test_vectors_with_a_nan_are_coded_like_the_oracle_does():
    """A sub-vector with a NaN has no nearest codebook entry; both sides leave it with entry 0."""
    w, M = cases()["byte-l2-m8"]
    print(f"[case] pq NaN vectors, workload={w.name} M={M}", flush=True)
    cb = synth.codebooks_from_rows(w.seed, w.base, M)
    g, o = make_pq_pair(w, M, cb)
    y = w.inserts[:40].copy()
    y[2, 0] = np.nan          # first sub-space only
    y[11, :] = np.nan
    g.add(dev(w.base[:1000])); o.add(w.base[:1000])
    g.add(dev(y)); o.add(y)
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    g.validate()
    assert_code_lists_equal(g, o)
    g.close()
