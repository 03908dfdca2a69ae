"""Sampled parity at the FULL size of configuration 4 (5 M x 768 unit vectors, inner product, 8,192
lists, T_m 128, nprobe 32, k 10, query batches of 1 to 64, seven search streams beside the data
stream under a mixed load of searches and inserts).  Blocks of 384 KiB, 43,000 of them, and the
widest vectors of any configuration are met at this size only.

The oracle builds the same index on the host.  Its own assignment pass would take the better part of
an hour for five million vectors of 768 dimensions against 8,192 centroids, so a double-precision
matrix product names the centroids that can win and the oracle's arithmetic decides among them; a
random sample of 50,000 vectors is assigned by the oracle itself and must agree.  Compared: the
length of every list, the contents of sampled lists bit for bit, queries at batches of 64 and of 1
within the tolerance, and all of it again after the mixed load.  No value here comes from the HIP
path."""
import numpy as np
import pytest
import torch

from oracle.oracle import OracleIndex
from paper_2408_02937_amd import synth
from tests.fullsize_common import check_assignment_on_sample, filtered_assignment, say
from tests.fullsize_gpu import build_pair, check_lengths_and_lists, check_queries
from tests.gpu_common import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def config4(request):
    torch.cuda.empty_cache()
    say(request, "configuration 4: drawing 5 M x 768")
    w = synth.config(4)
    print(f"[case] workload={w.name} seed={w.seed} n={len(w.base)}", flush=True)
    probe = OracleIndex(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=1)
    probe.set_centroids(w.centroids)
    say(request, "configuration 4: narrowing down the list of every vector (a minute of matrix products)")
    assign = np.empty(len(w.base), dtype=np.int32)
    piece = 1 << 19  # in pieces, so that a progress line appears every few seconds
    for lo in range(0, len(w.base), piece):
        assign[lo:lo + piece] = filtered_assignment(probe, w.metric, w.base[lo:lo + piece], w.centroids, rows_per_step=2048)
        say(request, f"configuration 4: {min(lo + piece, len(w.base))} vectors narrowed down")
    say(request, "configuration 4: the oracle assigns a sample of 50,000 vectors")
    check_assignment_on_sample(probe, w.base, assign, 50_000, seed=4)
    del probe
    g, o, data = build_pair(request, w, assign, n_resources=8,
                            cand=max(65536, 4 * w.nprobe * (len(w.base) // w.nlist + w.block_vecs)))
    yield w, g, o, data
    g.close()


def test_config4_lists(request, config4):
    w, g, o, _ = config4
    check_lengths_and_lists(request, w, g, o)


def test_config4_queries_batch_64_and_batch_1(request, config4):
    w, g, o, _ = config4
    check_queries(request, w, g, o, w.queries[:128], 64, "configuration 4, batch 64")
    check_queries(request, w, g, o, w.queries[128:136], 1, "configuration 4, batch 1")


def test_config4_mixed_load_on_seven_search_streams_then_parity(request, config4):
    """The configuration's launch shape: insert batches of 64 on the data stream while query batches
    of 1, 2, 4, ..., 64 go round seven search streams (about 70 % of the operations are queries); once
    all is quiet, lists and answers are the oracle's."""
    w, g, o, data = config4
    streams = [torch.cuda.Stream() for _ in range(7)]
    sizes = [1, 2, 4, 8, 16, 32, 64]
    nb, ib = 32, w.insert_batch
    ins = [dev(w.inserts[b * ib:(b + 1) * ib]) for b in range(nb)]
    Q = dev(w.queries[256:256 + 1024])
    cursor = step = 0
    for b in range(nb):
        g.add(ins[b], stream=data)
        for _ in range(8):  # 8 batches of 18 queries on average beside 64 inserted vectors: 70 % / 30 %
            n = sizes[step % 7]
            s_ = streams[step % 7]
            s_.synchronize()
            lo = cursor % (1024 - 64)
            g.search(Q[lo:lo + n], w.k, w.nprobe, stream=s_)
            cursor += n
            step += 1
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    o.add(w.inserts[:nb * ib])
    g.validate()
    assert np.array_equal(g.list_sizes(), o.list_sizes())
    say(request, "configuration 4: lists agree after the mixed load")
    check_queries(request, w, g, o, w.queries[2048:2048 + 64], 64, "configuration 4 after the mixed load")
