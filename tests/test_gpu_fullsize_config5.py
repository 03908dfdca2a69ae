"""Sampled parity at the FULL size of configuration 5 (20 M x 256, L2, 16,384 lists under a Zipf(1.1)
law, T_m 256, nprobe 64, k 50, batch 256), in the launch shape bench.py times.  Paths that exist only
at this size are met here: a list of millions of vectors and thousands of blocks (the upper segments
of its block table), scan budgets at their cap, work items of hot lists written by a whole workgroup.

The oracle builds the same index on the host; the list of every vector is known from how the set was
drawn, and a random sample of 100,000 vectors is assigned by the oracle itself and must agree.
Compared: the length of every list, the contents of sampled lists bit for bit (the longest among
them), 256 queries within the tolerance.  No value here comes from the HIP path."""
import numpy as np
import pytest
import torch

from paper_2408_02937_amd import synth
from tests.fullsize_common import check_assignment_on_sample, say
from tests.fullsize_gpu import build_pair, check_lengths_and_lists, check_queries
from tests.gpu_common import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def config5(request):
    say(request, "configuration 5: drawing 20 M x 256")
    w = synth.config(5)
    print(f"[case] workload={w.name} seed={w.seed} n={len(w.base)}", flush=True)
    assign = w.extra["base_component"].astype(np.int32)
    # a quarter of all vectors as candidates per query: the longest list holds a seventh of them
    g, o, data = build_pair(request, w, assign, cand=len(w.base) // 4)
    yield w, g, o, data, assign
    g.close()


def test_config5_assignment_by_construction_is_the_oracle_s(request, config5):
    w, g, o, _, assign = config5
    say(request, "configuration 5: the oracle assigns a sample of 100,000 vectors")
    n = check_assignment_on_sample(o, w.base, assign, 100_000, seed=5)
    say(request, f"configuration 5: {n} sampled vectors sit where the oracle puts them")


def test_config5_lists(request, config5):
    w, g, o, _, _ = config5
    sizes = check_lengths_and_lists(request, w, g, o)
    hot = int(sizes.argmax())
    blocks, runs, online = g.list_info(hot)
    assert blocks == (int(sizes[hot]) + w.block_vecs - 1) // w.block_vecs
    assert blocks > 8192, "the longest list should reach the upper segments of its block table"


def test_config5_queries_batch_256(request, config5):
    w, g, o, _, _ = config5
    check_queries(request, w, g, o, w.queries[:256], 256, "configuration 5, batch 256")


def test_config5_inserts_beside_searches_then_parity(request, config5):
    """The launch shape of the benchmark: batches of 1024 on the data stream, batches of 256 queries
    on several search streams beside them; once all is quiet, lists and answers are the oracle's."""
    w, g, o, data, _ = config5
    streams = [torch.cuda.Stream() for _ in range(4)]
    nb, ib = 16, w.insert_batch
    ins = [dev(w.inserts[b * ib:(b + 1) * ib]) for b in range(nb)]
    qs = [dev(w.queries[256 * (1 + b):256 * (2 + b)]) for b in range(4)]
    for b in range(nb):
        g.add(ins[b], stream=data)
        if b % 4 == 0:
            for t in streams:
                t.synchronize()
        g.search(qs[b % 4], w.k, w.nprobe, stream=streams[b % 4])
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    o.add(w.inserts[:nb * ib])
    g.validate()
    assert np.array_equal(g.list_sizes(), o.list_sizes())
    say(request, "configuration 5: lists agree after the concurrent inserts")
    check_queries(request, w, g, o, w.queries[2048:2048 + 64], 64, "configuration 5 after inserts")
