"""Sampled parity at the FULL size of configuration 3 (10 M x 96 unit vectors, inner product, 4,096
lists, T_m 256, nprobe 64, k 10, batch 128, four search streams beside the insert stream).

The oracle builds the same index on the host.  Its own assignment pass (one multiply-add chain per
vector and centroid) would take minutes for ten million vectors, so a double-precision matrix product
names the centroids that can win and the oracle's arithmetic decides among them; a random sample of
100,000 vectors is assigned by the oracle itself and must agree.  Compared: the length of every list,
the contents of sampled lists bit for bit, 256 queries within the tolerance.  No value here comes
from the HIP path."""
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
def config3(request):
    torch.cuda.empty_cache()
    say(request, "configuration 3: drawing 10 M x 96")
    w = synth.config(3)
    print(f"[case] workload={w.name} seed={w.seed} n={len(w.base)}", flush=True)
    probe = OracleIndex(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=1)
    probe.set_centroids(w.centroids)
    say(request, "configuration 3: narrowing down the list of every vector")
    assign = filtered_assignment(probe, w.metric, w.base, w.centroids)
    say(request, "configuration 3: the oracle assigns a sample of 100,000 vectors")
    check_assignment_on_sample(probe, w.base, assign, 100_000, seed=3)
    del probe
    g, o, data = build_pair(request, w, assign, cand=max(65536, 4 * w.nprobe * (len(w.base) // w.nlist + w.block_vecs)))
    yield w, g, o, data
    g.close()


def test_config3_lists(request, config3):
    w, g, o, _ = config3
    check_lengths_and_lists(request, w, g, o)


def test_config3_queries_batch_128(request, config3):
    w, g, o, _ = config3
    check_queries(request, w, g, o, w.queries[:256], 128, "configuration 3, batch 128")


def test_config3_four_search_streams_beside_inserts_then_parity(request, config3):
    w, g, o, data = config3
    streams = [torch.cuda.Stream() for _ in range(4)]
    nb, ib = 16, w.insert_batch
    ins = [dev(w.inserts[b * ib:(b + 1) * ib]) for b in range(nb)]
    qs = [dev(w.queries[128 * (2 + b):128 * (3 + b)]) for b in range(4)]
    for b in range(nb):
        g.add(ins[b], stream=data)
        for s_, q_ in zip(streams, qs):
            s_.synchronize()
            g.search(q_, w.k, w.nprobe, stream=s_)
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    o.add(w.inserts[:nb * ib])
    g.validate()
    assert np.array_equal(g.list_sizes(), o.list_sizes())
    check_queries(request, w, g, o, w.queries[1024:1024 + 128], 128, "configuration 3 after inserts")
