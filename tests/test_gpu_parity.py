"""HIP path against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import assert_lists_equal, dev, make_pair, scan_modes
from tests.helpers import assert_topk_matches, RTOL

pytestmark = pytest.mark.gpu



def workloads():
    return {
        "tiny-l2": synth.config(1),
        "byte-l2": synth.byte_valued_l2("byte-small", 21, n_base=30_000, n_centres=40, nlist=96,
                                        block_vecs=128, n_queries=300, n_inserts=3_000, insert_batch=64,
                                        nprobe=12, k=100),
        "unit-ip": synth.unit_ip("ip-small", 22, d=96, n_base=40_000, n_centres=300, nlist=128,
                                 block_vecs=256, n_queries=300, n_inserts=2_048, insert_batch=512,
                                 nprobe=16, k=10),
        "zipf-l2": synth.skewed_l2("zipf-small", 23, d=64, n_base=60_000, nlist=256, block_vecs=64,
                                   n_queries=256, n_inserts=4_096, insert_batch=1024, nprobe=16, k=50),
    }


@pytest.fixture(scope="module", params=list(workloads().keys()))
def loaded(request):
    """Base set bulk-loaded in one add, then the insert stream in its batches."""
    w = workloads()[request.param]
    print(f"[case] workload={w.name} seed={w.seed}", flush=True)
    g, o = make_pair(w)
    g.set_param("use_mfma", 2)  # every batch of 32 rows or more goes through the matrix-core filter
    g.add(dev(w.base))
    o.add(w.base)
    bounds = [len(w.base)]
    for b in range(0, len(w.inserts), w.insert_batch):
        chunk = w.inserts[b:b + w.insert_batch]
        g.add(dev(chunk))
        o.add(chunk)
        bounds.append(bounds[-1] + len(chunk))
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    yield w, g, o, np.array(bounds[:-1])
    g.close()


def test_assignment_is_bit_exact(loaded):
    w, g, o, _ = loaded
    y = np.concatenate([w.inserts, w.queries])
    got = g.assign(dev(y)).cpu().numpy()
    assert np.array_equal(got, o.assign(y))


def test_list_contents_and_block_structure(loaded):
    w, g, o, bounds = loaded
    g.validate()
    assert_lists_equal(g, o, bounds)


@pytest.mark.parametrize("name,mfma,max_add_batch", [("tiny-l2", 0, 65536), ("zipf-l2", 2, 65536),
                                                     ("zipf-l2", 0, 1000), ("unit-ip", 2, 4096)])
def test_ordered_insertion_gives_the_oracle_s_sequences(name, mfma, max_add_batch):
    """With positions handed out in the order of the batch ("ordered_add") every
    list holds, entry by entry, what inserting the vectors one at a time gives:
    the oracle's sequences, not merely its sets.  The bulk load is cut into
    rounds of max_add_batch inside the library; the skewed set puts hundreds of
    vectors of one batch, and several new blocks, into one list."""
    w = workloads()[name]
    print(f"[case] ordered insertion, workload={w.name} use_mfma={mfma} max_add_batch={max_add_batch}", flush=True)
    g, o = make_pair(w, max_add_batch=max_add_batch)
    g.set_param("use_mfma", mfma)
    g.set_param("ordered_add", 1)
    g.add(dev(w.base))
    o.add(w.base)
    for b in range(0, len(w.inserts), w.insert_batch):
        chunk = w.inserts[b:b + w.insert_batch]
        g.add(dev(chunk))
        o.add(chunk)
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    g.validate()
    assert np.array_equal(g.list_sizes(), o.list_sizes())
    for k in range(g.nlist):
        gi, gx = g.list_export(k)
        oi, ox = o.list_export(k)
        assert np.array_equal(gi.cpu().numpy(), oi), f"list {k}: id sequence differs"
        assert np.array_equal(gx.cpu().numpy().view(np.uint32), ox.view(np.uint32)), f"list {k}: vectors differ"
    # and a search over them is the oracle's
    q = w.queries[:64]
    d, i = g.search(dev(q), w.k, w.nprobe)
    torch.cuda.synchronize()
    rd, ri = o.search(q, w.k, w.nprobe)
    assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd, ri, RTOL)
    g.close()


def test_probe_selection_is_bit_exact(loaded):
    w, g, o, _ = loaded
    for nprobe in (1, w.nprobe, min(w.nlist, 64)):
        got = g.probe(dev(w.queries[:256]), nprobe).cpu().numpy()
        assert np.array_equal(got, o.probe(w.queries[:256], nprobe)), f"nprobe={nprobe}"


@pytest.mark.parametrize("batch", [1, 7, 256])
def test_search_matches_oracle(loaded, batch):
    w, g, o, _ = loaded
    q = w.queries[:batch]
    rd, ri = o.search(q, w.k, w.nprobe)
    for mode in scan_modes(g):
        d, i = g.search(dev(q), w.k, w.nprobe)
        torch.cuda.synchronize()
        assert g.poll_error() == 0
        assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6,
                            what=f"{w.name} batch {batch} scan_mfma {mode}")


def test_long_scans_that_take_work_from_other_dies_match_the_oracle(loaded):
    """A scan that the library takes for a long one lets a die that has run out of work items take
    items from the back of another die's share (matrix-core scan).  Every request is made to count as
    long here; with and without the taking the answers are the oracle's, and the same bits."""
    w, g, o, _ = loaded
    q = w.queries[:256]
    rd, ri = o.search(q, w.k, w.nprobe)
    got = {}
    try:
        g.set_param("scan_exclusive_pairs", 1)
        g.set_param("scan_exclusive_bytes", 1)
        g.set_param("scan_mfma", 2)
        for steal in (1, 0):
            g.set_param("scan_steal", steal)
            for rep in range(3):  # which die finishes first differs from run to run
                d, i = g.search(dev(q), w.k, w.nprobe)
                torch.cuda.synchronize()
                assert g.poll_error() == 0
                d, i = d.cpu().numpy(), i.cpu().numpy()
                assert_topk_matches(w.metric, d, i, rd, ri, rtol=RTOL, atol=1e-6, what=f"{w.name} steal {steal} run {rep}")
                if got:
                    assert np.array_equal(i, got["i"]) and np.array_equal(d.view(np.uint32), got["d"].view(np.uint32))
                else:
                    got = {"d": d, "i": i}
    finally:
        g.set_param("scan_steal", 1)
        g.set_param("scan_mfma", 1)
        g.set_param("scan_exclusive_pairs", 4096)
        g.set_param("scan_exclusive_bytes", 16 << 30)


def test_search_all_lists_and_large_k(loaded):
    w, g, o, _ = loaded
    nprobe = min(w.nlist, 64)
    q = w.queries[:32]
    rd, ri = o.search(q, 128, nprobe)
    for mode in scan_modes(g):
        d, i = g.search(dev(q), 128, nprobe)
        torch.cuda.synchronize()
        assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6,
                            what=f"scan_mfma {mode}")


@pytest.mark.parametrize("mfma", [0, 2])
def test_many_results_and_many_probes(mfma):
    """k and nprobe beyond what is put in order by ranking (256 entries): the
    sorting network with its padding, for the probe lists and for the results."""
    w = synth.gaussian_l2("wide", 24, d=16, n_base=20_000, n_centres=50, nlist=400, block_vecs=64, n_queries=64,
                          n_inserts=10, nprobe=300, k=700)
    print(f"[case] k={w.k} nprobe={w.nprobe} nlist={w.nlist} use_mfma={mfma}", flush=True)
    g, o = make_pair(w, max_k=1024, max_nprobe=400, max_batch=64)
    g.set_param("use_mfma", mfma)
    g.add(dev(w.base)); o.add(w.base)
    for nprobe, k in ((300, 700), (257, 1024), (400, 300)):
        q = w.queries[:40]
        assert np.array_equal(g.probe(dev(q), nprobe).cpu().numpy(), o.probe(q, nprobe))
        rd, ri = o.search(q, k, nprobe)
        for mode in scan_modes(g):
            d, i = g.search(dev(q), k, nprobe)
            torch.cuda.synchronize()
            assert g.poll_error() == 0
            assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6,
                                what=f"nprobe {nprobe} k {k} scan_mfma {mode}")
    g.close()


def test_integer_valued_distances_are_exact():
    """Byte-valued data: every partial sum is an integer below 2^24, so fp32 is
    exact and ids (ties by id included) and distances must equal the oracle's."""
    w = workloads()["byte-l2"]
    g, o = make_pair(w)
    base = np.concatenate([w.base, w.base[:500]])      # duplicates: exact ties
    g.add(dev(base)); o.add(base)
    q = w.queries[:256]
    rd, ri = o.search(q, w.k, w.nprobe)
    for mode in scan_modes(g):  # the norm form of the matrix cores is exact on such data as well
        d, i = g.search(dev(q), w.k, w.nprobe)
        torch.cuda.synchronize()
        assert np.array_equal(i.cpu().numpy(), ri), f"scan_mfma {mode}"
        assert np.array_equal(d.cpu().numpy().astype(np.float64), rd), f"scan_mfma {mode}"
        d, i = g.search(dev(base[7:8]), 2, w.nprobe)      # both copies of a duplicated row, lower id first
        assert i.cpu().numpy()[0].tolist() == [7, len(w.base) + 7] and d.cpu().numpy()[0].tolist() == [0.0, 0.0]
    g.close()


@pytest.mark.parametrize("metric", ["l2", "ip"])
def test_many_lists_assignment_and_probes(metric):
    """More centroids than one pass of a workgroup covers: each thread of the
    coarse kernel walks several centroid rows (nlist 16384, as in the largest
    configuration), for a big insertion batch and for a query batch."""
    rng = np.random.default_rng(31)
    d, nlist = 8, 16384
    C = rng.standard_normal((nlist, d), dtype=np.float32)
    w = synth.Workload("many-lists", metric, d, nlist, 64, 64, 10, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 0)
    g, o = make_pair(w, pool_blocks=20000, candidates_per_query=4096)
    y = rng.standard_normal((20000, d), dtype=np.float32)
    for filt in (2, 0):  # with and without the matrix-core filter in front of the exact arithmetic
        g.set_param("use_mfma", filt)
        assert np.array_equal(g.assign(dev(y)).cpu().numpy(), o.assign(y)), f"filter={filt}"
        for nq in (3, 256):
            assert np.array_equal(g.probe(dev(y[:nq]), 64).cpu().numpy(), o.probe(y[:nq], 64)), f"filter={filt}"
    g.set_param("use_mfma", 1)
    g.add(dev(y)); o.add(y)
    g.validate()
    assert np.array_equal(g.list_sizes(), o.list_sizes())
    dd, ii = g.search(dev(y[:256]), 10, 64)
    rd, ri = o.search(y[:256], 10, 64)
    assert_topk_matches(metric, dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6)
    g.close()


@pytest.mark.parametrize("metric", ["l2", "ip"])
def test_coarse_filter_cannot_separate_near_duplicate_centroids(metric):
    """1500 of 2048 centroids differ only in the last bits: the fp32 filter of a
    large batch cannot tell them apart (more candidates than its refinement
    holds), so assignment and probe selection must come out of the exact
    arithmetic alone, ties to the lowest index."""
    rng = np.random.default_rng(77)
    d, nlist = 32, 2048
    C = rng.standard_normal((nlist, d), dtype=np.float32)
    dup = rng.permutation(nlist)[:1500]
    C[dup] = C[dup[0]] * (1 + rng.integers(-2, 3, (1500, d)).astype(np.float32) * np.float32(2.0 ** -23))
    C[dup[100:140]] = C[dup[0]]  # and some exact copies
    w = synth.Workload("near-dup-centroids", metric, d, nlist, 64, 16, 10, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 0)
    g, o = make_pair(w, pool_blocks=8000, candidates_per_query=8192)
    g.set_param("use_mfma", 2)
    y = np.concatenate([C[dup[0]] + 0.05 * rng.standard_normal((3000, d)),
                        rng.standard_normal((3000, d))]).astype(np.float32)
    assert np.array_equal(g.assign(dev(y)).cpu().numpy(), o.assign(y))
    q = np.concatenate([y[:100], y[3000:3100]])
    for nprobe in (1, 16, 64):
        assert np.array_equal(g.probe(dev(q), nprobe).cpu().numpy(), o.probe(q, nprobe)), f"nprobe={nprobe}"
    g.close()


def test_coarse_filter_under_cancellation():
    """Vectors and centroids far from the origin, close to each other: the
    norm expansion the filter uses loses every significant digit of the
    distances, its error band covers most centroids, and the decisions must still
    be those of the exact arithmetic."""
    rng = np.random.default_rng(78)
    d, nlist = 64, 512
    C = (1000.0 + rng.standard_normal((nlist, d))).astype(np.float32)
    w = synth.Workload("far-from-origin", "l2", d, nlist, 64, 16, 10, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 0)
    g, o = make_pair(w, pool_blocks=4000, candidates_per_query=8192)
    g.set_param("use_mfma", 2)
    y = (1000.0 + rng.standard_normal((4096, d))).astype(np.float32)
    assert np.array_equal(g.assign(dev(y)).cpu().numpy(), o.assign(y))
    for nprobe in (1, 16, 64):
        assert np.array_equal(g.probe(dev(y[:256]), nprobe).cpu().numpy(), o.probe(y[:256], nprobe))
    g.add(dev(y)); o.add(y)
    assert_lists_equal(g, o)
    g.close()


@pytest.mark.parametrize("shape", [
    dict(d=4, nlist=100, block_vecs=64, metric="l2", nprobe=100, k=1, batch=77),
    dict(d=20, nlist=37, block_vecs=192, metric="ip", nprobe=9, k=1000, batch=5),
    dict(d=260, nlist=50, block_vecs=128, metric="l2", nprobe=50, k=33, batch=130),
])
@pytest.mark.parametrize("mfma", [1, 2])
def test_odd_shapes(shape, mfma):
    """Dimensions that are not a multiple of the scan's pipeline depth (nor of the 32 coordinates the
    matrix-core filter takes per step), blocks of three groups, list counts that are no power of two
    (nor a multiple of the filter's 128-centroid tiles), every list probed, k = 1 and k near its
    maximum; with the coarse filter left to the library's rule and forced on."""
    d, nlist, metric = shape["d"], shape["nlist"], shape["metric"]
    rng = np.random.default_rng(100 + d)
    C = rng.standard_normal((nlist, d)).astype(np.float32)
    w = synth.Workload("odd", metric, d, nlist, shape["block_vecs"], shape["nprobe"], shape["k"],
                       np.zeros((0, d), np.float32), C, np.zeros((0, d), np.float32),
                       np.zeros((0, d), np.float32), 1, 0)
    g, o = make_pair(w, pool_blocks=600, max_k=1024, max_nprobe=128, candidates_per_query=30000)
    g.set_param("use_mfma", mfma)
    y = (C[rng.integers(0, nlist, 25000)] + 0.3 * rng.standard_normal((25000, d))).astype(np.float32)
    for b in range(0, len(y), 7000):  # ragged batches
        g.add(dev(y[b:b + 7000])); o.add(y[b:b + 7000])
    g.validate()
    assert_lists_equal(g, o)
    q = (C[rng.integers(0, nlist, shape["batch"])] + 0.3 * rng.standard_normal((shape["batch"], d))).astype(np.float32)
    rd, ri = o.search(q, shape["k"], shape["nprobe"])
    for mode in scan_modes(g):
        dd, ii = g.search(dev(q), shape["k"], shape["nprobe"])
        assert_topk_matches(metric, dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6,
                            what=f"scan_mfma {mode}")
    g.close()


@pytest.mark.parametrize("d,metric", [(1024, "l2"), (2048, "ip"), (2048, "l2")])
def test_widest_vectors(d, metric):
    """The widest vectors the configuration accepts (d up to 2048): the coarse kernel's tile of vectors
    and the scans' tiles of queries have to fit LDS; assignment, lists, probes and searches as ever."""
    rng = np.random.default_rng(d)
    nlist = 48
    C = rng.standard_normal((nlist, d)).astype(np.float32)
    w = synth.Workload("wide-vectors", metric, d, nlist, 64, 8, 10, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 0)
    g, o = make_pair(w, pool_blocks=200, candidates_per_query=6000)
    y = (C[rng.integers(0, nlist, 3000)] + 0.3 * rng.standard_normal((3000, d))).astype(np.float32)
    for use_mfma in (0, 2):
        g.set_param("use_mfma", use_mfma)
        assert np.array_equal(g.assign(dev(y[:300])).cpu().numpy(), o.assign(y[:300])), f"use_mfma {use_mfma}"
    g.add(dev(y)); o.add(y)
    g.validate()
    assert_lists_equal(g, o)
    q = (C[rng.integers(0, nlist, 70)] + 0.3 * rng.standard_normal((70, d))).astype(np.float32)
    for nq in (1, 70):
        assert np.array_equal(g.probe(dev(q[:nq]), 8).cpu().numpy(), o.probe(q[:nq], 8))
        rd, ri = o.search(q[:nq], 10, 8)
        for mode in scan_modes(g):
            dd, ii = g.search(dev(q[:nq]), 10, 8)
            assert g.poll_error() == 0
            assert_topk_matches(metric, dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6,
                                what=f"d {d} batch {nq} scan_mfma {mode}")
    g.close()


def test_loose_bound_and_worst_first_records():
    """The pruning bound of a query comes from the head of its nearest list.  Here that head is 600
    decoys far from the query, so every candidate passes the bound, and the true neighbours sit
    in another list ordered worst first: the selection has to take tens of thousands of survivor
    records through LDS, renewing its limit as better ones keep coming."""
    rng = np.random.default_rng(5)
    d, nlist, n_near = 16, 8, 30000
    C = np.zeros((nlist, d), np.float32)
    C[1, 0] = 2.0
    C[2:, 1] = 50.0 + np.arange(nlist - 2)  # far away, probed but empty
    w = synth.Workload("loose-bound", "l2", d, nlist, 64, nlist, 100, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 0)
    g, o = make_pair(w, pool_blocks=1000, candidates_per_query=40000)
    decoys = np.zeros((600, d), np.float32)
    decoys[:, 0] = -0.9
    decoys += 0.01 * rng.standard_normal((600, d)).astype(np.float32)
    near = 0.001 * rng.standard_normal((n_near, d)).astype(np.float32)
    near[:, 0] = 1.02 + 0.28 * (1.0 - np.arange(n_near, dtype=np.float32) / n_near)  # worst first
    for part in (decoys, near):
        g.add(dev(part)); o.add(part)
    assert np.array_equal(g.list_sizes(), o.list_sizes()) and g.list_sizes()[0] == 600
    q = np.zeros((3, d), np.float32)
    q[:, 0] = (0.95, 0.9, 0.8)
    for k in (1, 100):
        rd, ri = o.search(q, k, nlist)
        for mode in scan_modes(g):
            dd, ii = g.search(dev(q), k, nlist)
            assert_topk_matches("l2", dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6,
                                what=f"k {k} scan_mfma {mode}")
    g.close()


def test_k_larger_than_a_query_has_candidates():
    """Fewer candidates than k (and than the bound's sample): everything is kept, the rest of the
    row is padding."""
    rng = np.random.default_rng(6)
    d, nlist = 8, 16
    C = rng.standard_normal((nlist, d)).astype(np.float32)
    w = synth.Workload("few-candidates", "ip", d, nlist, 64, 2, 128, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 0)
    g, o = make_pair(w, pool_blocks=200, candidates_per_query=4096)
    y = rng.standard_normal((700, d)).astype(np.float32)
    g.add(dev(y)); o.add(y)
    q = rng.standard_normal((40, d)).astype(np.float32)
    rd, ri = o.search(q, 128, 2)
    assert (ri == -1).any()  # some query does run short
    for mode in scan_modes(g):
        dd, ii = g.search(dev(q), 128, 2)
        assert_topk_matches("ip", dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6,
                            what=f"scan_mfma {mode}")
    g.close()


def test_massive_ties_fall_back_to_in_place_selection():
    """Thousands of identical vectors: every candidate ties at the k-th score, more
    than the selection keeps in LDS, so the lowest ids must win."""
    rng = np.random.default_rng(9)
    d, nlist = 16, 4
    C = rng.standard_normal((nlist, d), dtype=np.float32)
    w = synth.Workload("ties", "l2", d, nlist, 64, 4, 100, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 0)
    g, o = make_pair(w, pool_blocks=400, candidates_per_query=20000)
    same = np.repeat(C[1:2] + np.float32(0.25), 9000, axis=0)
    other = (C[rng.integers(0, nlist, 3000)] + rng.standard_normal((3000, d))).astype(np.float32)
    ids = rng.permutation(12000).astype(np.int64)
    y = np.concatenate([same, other])
    g.add(dev(y), dev(ids)); o.add(y, ids)
    q = np.concatenate([C[1:2] + np.float32(0.25), other[:7]])
    rd, ri = o.search(q, 100, 4)
    for mode in scan_modes(g):
        dd, ii = g.search(dev(q), 100, 4)
        assert np.array_equal(ii.cpu().numpy()[0], ri[0]) and np.all(dd.cpu().numpy()[0] == 0.0), f"scan_mfma {mode}"
        assert_topk_matches("l2", dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6,
                            what=f"scan_mfma {mode}")
    g.close()


@pytest.mark.parametrize("offset", [30.0, 1000.0])
def test_scan_under_cancellation(offset):
    """Squared distances of vectors far from the origin and close to each other.  On the matrix cores
    the scan scores |x|^2 + |q|^2 - 2 <x, q>, which loses the significant digits of such distances
    (at offset 1000 every digit: norms of 6.4e7 against distances of 0.6); the margin it keeps and the
    direct-form scores the selection gives its finalists must return the oracle's answer within the
    tolerance all the same.  Tiles of one query and of many (a batch of 1 and of 200 that share lists)."""
    rng = np.random.default_rng(1234)
    d, nlist = 64, 32
    C = (offset + rng.standard_normal((nlist, d))).astype(np.float32)
    w = synth.Workload("scan-cancellation", "l2", d, nlist, 64, 8, 20, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 0)
    g, o = make_pair(w, pool_blocks=1200, candidates_per_query=60000)
    y = (C[rng.integers(0, nlist, 50000)] + 0.1 * rng.standard_normal((50000, d))).astype(np.float32)
    g.add(dev(y)); o.add(y)
    assert np.array_equal(g.list_sizes(), o.list_sizes())
    q = (C[rng.integers(0, nlist, 200)] + 0.1 * rng.standard_normal((200, d))).astype(np.float32)
    for nq in (1, 200):
        rd, ri = o.search(q[:nq], 20, 8)
        for mode in scan_modes(g):
            dd, ii = g.search(dev(q[:nq]), 20, 8)
            assert g.poll_error() == 0
            assert_topk_matches("l2", dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6,
                                what=f"offset {offset} batch {nq} scan_mfma {mode}")
    g.close()


def test_caller_ids_and_ragged_tail():
    """Caller-supplied ids; list lengths that end inside a 64-vector group and
    inside a block; a batch that opens several blocks for one list."""
    rng = np.random.default_rng(5)
    d, nlist, T = 8, 3, 64
    C = np.eye(nlist, d, dtype=np.float32) * 4
    w = synth.Workload("ragged", "l2", d, nlist, T, 3, 10, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 0)
    g, o = make_pair(w, pool_blocks=64, candidates_per_query=2000)
    sizes = [1, 63, 64, 65, 200, 1]
    next_id = 10_000
    for s, n in enumerate(sizes):
        comp = rng.integers(0, nlist, size=n) if s != 4 else np.zeros(n, dtype=np.int64)
        y = (C[comp] + 0.3 * rng.standard_normal((n, d))).astype(np.float32)
        ids = np.arange(next_id, next_id + n, dtype=np.int64)[::-1].copy()   # descending on purpose
        next_id += n
        g.add(dev(y), dev(ids)); o.add(y, ids)
    g.validate()
    assert_lists_equal(g, o)
    q = (C[rng.integers(0, nlist, size=40)] + 0.3 * rng.standard_normal((40, d))).astype(np.float32)
    for nprobe in (1, 3):
        dd, ii = g.search(dev(q), 10, nprobe)
        rd, ri = o.search(q, 10, nprobe)
        assert_topk_matches("l2", dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6)
    g.close()


def test_empty_index_short_lists_and_errors():
    d, nlist = 4, 4
    C = np.eye(4, dtype=np.float32)
    w = synth.Workload("empty", "ip", d, nlist, 64, 4, 3, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 0)
    g = rtams.Index(d, nlist, "ip", 64, pool_blocks=8, max_batch=4, max_k=8, max_nprobe=4,
                    candidates_per_query=256, n_resources=2)
    q = dev(np.ones((1, d), np.float32))
    with pytest.raises(rtams.RtamsError) as e:
        g.search(q, 3, 4)
    assert e.value.code == rtams.ESTATE
    g.set_centroids(dev(C))
    dd, ii = g.search(q, 3, 4)                                   # nothing inserted yet
    assert ii.cpu().numpy().tolist() == [[-1, -1, -1]] and np.all(np.isneginf(dd.cpu().numpy()))
    g.add(dev(C[:2]))
    dd, ii = g.search(dev(np.array([[1, 0, 0, 0]], np.float32)), 3, 4)
    assert ii.cpu().numpy().tolist() == [[0, 1, -1]]
    assert dd.cpu().numpy()[0, :2].tolist() == [1.0, 0.0] and np.isneginf(dd.cpu().numpy()[0, 2])
    for bad in (dict(k=9, nprobe=1), dict(k=1, nprobe=5), dict(k=0, nprobe=1)):
        with pytest.raises(rtams.RtamsError) as e:
            g.search(q, bad["k"], bad["nprobe"])
        assert e.value.code == rtams.EINVAL
    with pytest.raises(rtams.RtamsError) as e:
        g.search(dev(np.ones((5, d), np.float32)), 1, 1)        # nq > max_batch
    assert e.value.code == rtams.EINVAL
    g.close()


@pytest.mark.parametrize("mfma", [0, 2])
def test_vectors_whose_scores_do_not_compare_go_to_the_first_list(mfma):
    """A vector with a NaN coordinate has no nearest centroid: no score is better
    than another.  Both sides then leave it with the first centroid (the running
    best starts there and is never beaten), and every other vector of the batch is
    placed as usual."""
    w = workloads()["tiny-l2"]
    print(f"[case] NaN vectors in a batch, use_mfma={mfma}", flush=True)
    g, o = make_pair(w)
    g.set_param("use_mfma", mfma)
    y = w.inserts[:48].copy()
    y[3, 5] = np.nan
    y[17, :] = np.nan
    y[40, 0] = np.nan
    assert o.assign(y)[[3, 17, 40]].tolist() == [0, 0, 0]
    assert np.array_equal(g.assign(dev(y)).cpu().numpy(), o.assign(y))
    g.add(dev(w.base[:2000])); o.add(w.base[:2000])
    g.add(dev(y)); o.add(y)
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    g.validate()
    assert np.array_equal(g.list_sizes(), o.list_sizes())
    ids = g.list_export(0)[0].cpu().numpy()
    assert {2003, 2017, 2040} <= set(ids.tolist())
    g.close()


@pytest.mark.parametrize("mfma", [0, 2])
def test_queries_whose_scores_do_not_compare_disturb_nobody(loaded, mfma):
    """Queries with a NaN coordinate have no nearest anything; they get some rows of
    valid ids (or padding) back, and the other queries of the batch their exact answers."""
    w, g, o, _ = loaded
    g.set_param("use_mfma", mfma)
    q = w.queries[:40].copy()
    q[5, 1] = np.nan
    q[33, :] = np.nan
    d, i = g.search(dev(q), w.k, w.nprobe)
    torch.cuda.synchronize()
    g.set_param("use_mfma", 2)
    assert g.poll_error() == 0
    d, i = d.cpu().numpy(), i.cpu().numpy()
    good = np.ones(40, bool); good[[5, 33]] = False
    rd, ri = o.search(q[good], w.k, w.nprobe)
    assert_topk_matches(w.metric, d[good], i[good], rd, ri, rtol=RTOL, atol=1e-6)
    known = set(np.concatenate([g.list_export(k)[0].cpu().numpy() for k in range(g.nlist)]).tolist()) | {-1}
    assert set(i[~good].ravel().tolist()) <= known


def test_pool_exhaustion_is_refused_before_anything_is_enqueued():
    d, nlist, T = 4, 2, 64
    C = np.eye(2, 4, dtype=np.float32)
    g = rtams.Index(d, nlist, "ip", T, pool_blocks=3, max_batch=4, max_k=8, max_nprobe=2,
                    candidates_per_query=1024, n_resources=2)
    g.set_centroids(dev(C))
    total = g.pool_stats().blocks_total
    g.add(dev(np.repeat(C[:1], T * (total - 2), axis=0)))       # all but two blocks
    with pytest.raises(rtams.RtamsError) as e:
        g.add(dev(np.repeat(C[1:], 2 * T + 1, axis=0)))         # needs three
    assert e.value.code == rtams.EPOOL
    st = g.pool_stats()
    assert st.ntotal == T * (total - 2) and st.blocks_in_use == total - 2 and g.poll_error() == 0
    g.validate()
    g.close()


def test_add_learns_the_blocks_left_from_the_device_s_reports_without_waiting():
    """Every add counts the blocks it may open at most (one per list it might touch, plus the full
    ones) against the blocks left.  Small batches over many lists open far fewer than that, so the
    running count falls short long before the pool does; the blocks in use that the device reports
    at every publication then put it right, and the call never has to wait for the data stream.
    The lists are the oracle's afterwards; a pool that really is full is still refused."""
    w = synth.gaussian_l2("pool-bound", 77, d=16, n_base=6400, n_centres=32, nlist=64, block_vecs=64,
                          n_queries=8, n_inserts=64)
    # 6,400 vectors over 64 lists fill about 130 blocks; 100 batches of 64 may open 65 each by the count
    g, o = make_pair(w, pool_blocks=400, max_batch=8, max_k=16, max_nprobe=8, candidates_per_query=8192)
    s = torch.cuda.Stream()
    for lo in range(0, len(w.base), 64):
        g.add(dev(w.base[lo:lo + 64]), stream=s)
        s.synchronize()  # what the device reported is there for the next call to read
    o.add(w.base)
    st = g.pool_stats()
    assert st.add_waits == 0, "an add waited for the data stream although the device had reported enough blocks left"
    assert st.blocks_in_use == o.blocks_in_use and st.blocks_in_use < 200
    assert_lists_equal(g, o)
    g.validate()
    # batches enqueued back to back: the calls not yet published count with what they may open, so the
    # estimate can only fall short (a wait), never let a batch through that does not fit
    more = synth.gaussian_l2("pool-bound-more", 78, d=16, n_base=64 * 40, n_centres=32, nlist=64, block_vecs=64,
                             n_queries=8, n_inserts=64)
    for lo in range(0, len(more.base), 64):  # 40 batches need some 40 blocks of the 250 left: none may be refused
        g.add(dev(more.base[lo:lo + 64]), stream=s)
    s.synchronize()
    assert g.poll_error() == 0
    o.add(more.base)
    st2 = g.pool_stats()
    assert st2.blocks_in_use == o.blocks_in_use
    assert_lists_equal(g, o)
    g.validate()
    g.close()


def test_centroids_set_twice_replace_every_copy_the_kernels_read():
    """Before the first vector is in, the centroids may be set again.  The library keeps them row by
    row (exact rescoring), transposed (the exact coarse kernel), as bf16 halves and as squared norms
    (the matrix-core filter): assignments and probe sets must follow the SECOND set on every path,
    exact kernel alone and filter in front of it."""
    w = synth.gaussian_l2("twice", 91, d=48, n_base=3000, n_centres=40, nlist=130, block_vecs=64,
                          n_queries=64, n_inserts=64)
    g, o = make_pair(w, max_batch=64, max_k=16, max_nprobe=16)
    first = np.ascontiguousarray(w.base[::-1][:w.nlist] * 3.0 + 1.0)  # nothing like the real ones
    g.set_centroids(dev(first))
    g.set_centroids(dev(w.centroids))
    ref_assign = o.assign(w.base[:2000])
    ref_probe = o.probe(w.queries, 16)
    for mfma in (0, 2):
        g.set_param("use_mfma", mfma)
        assert np.array_equal(g.assign(dev(w.base[:2000])).cpu().numpy(), ref_assign), f"use_mfma={mfma}: assignment"
        assert np.array_equal(g.assign(dev(w.base[:3])).cpu().numpy(), ref_assign[:3]), f"use_mfma={mfma}: small batch"
        assert np.array_equal(g.probe(dev(w.queries), 16).cpu().numpy(), ref_probe), f"use_mfma={mfma}: probes"
        assert np.array_equal(g.probe(dev(w.queries[:1]), 16).cpu().numpy(), ref_probe[:1]), f"use_mfma={mfma}: one query"
    g.set_param("use_mfma", 1)
    g.add(dev(w.base))
    o.add(w.base)
    with pytest.raises(rtams.RtamsError) as e:  # once vectors are in, the centroids stay
        g.set_centroids(dev(first))
    assert e.value.code == rtams.ESTATE
    assert_lists_equal(g, o)
    g.close()


def test_timed_scans_are_counted_by_the_kernel_that_ran(loaded):
    """The benchmark names the scan kernel of its roofline from these counts."""
    w, g, o, _ = loaded
    q = dev(w.queries[:64])
    g.scan_kernels(reset=True)
    g.scan_time(reset=True)
    g.set_param("profile_scan", 1)
    try:
        for mode, name in ((2, "k_scan_mm"), (0, "k_scan")):
            g.set_param("scan_mfma", mode)
            for _ in range(3):
                g.search(q, w.k, w.nprobe)
            torch.cuda.synchronize()
            got = g.scan_kernels(reset=True)
            assert got[name] == 3 and sum(got.values()) == 3, (mode, got)
        ms, n = g.scan_time(reset=True)
        assert n == 6 and ms > 0.0
    finally:
        g.set_param("profile_scan", 0)
        g.set_param("scan_mfma", 1)
    g.search(q, w.k, w.nprobe)  # not timed: not counted
    torch.cuda.synchronize()
    assert sum(g.scan_kernels().values()) == 0
