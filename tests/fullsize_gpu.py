"""Steps the full-size parity files share: build the pair of indexes, compare lists, compare queries."""
import numpy as np
import pytest
import torch

from paper_2408_02937_amd import rtams, synth
from oracle.oracle import OracleIndex
from tests.fullsize_common import compare_lists, say
from tests.gpu_common import dev, scan_modes
from tests.helpers import ATOL, RTOL, assert_topk_matches


def build_pair(request, w, assign, cand, rearrange_threshold=0, spare_blocks=64, n_resources=5):
    n_all = len(w.base) + len(w.inserts)
    pool_blocks = n_all // w.block_vecs + 2 * w.nlist + spare_blocks
    g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=pool_blocks,
                    rearrange_threshold=rearrange_threshold, n_resources=n_resources, max_batch=256, max_k=64,
                    max_nprobe=64, max_add_batch=65536, candidates_per_query=cand)
    g.set_centroids(dev(w.centroids))
    o = OracleIndex(w.d, w.nlist, w.metric, w.block_vecs, rearrange_threshold=0, pool_blocks=pool_blocks)
    o.set_centroids(w.centroids)
    data = torch.cuda.Stream()
    say(request, f"{w.name}: bulk load of {len(w.base)} vectors on the GPU")
    for lo in range(0, len(w.base), 1 << 22):  # in pieces, so the whole set need not sit in HBM twice
        part = dev(w.base[lo:lo + (1 << 22)])
        g.add(part, stream=data)
        data.synchronize()
        del part
    say(request, f"{w.name}: the oracle takes the same vectors")
    o.add(w.base, assign=assign)
    return g, o, data


def check_lengths_and_lists(request, w, g, o, n_lists=14):
    g.validate()
    assert g.poll_error() == 0
    sizes = g.list_sizes()
    assert np.array_equal(sizes, o.list_sizes()), "list lengths differ from the oracle's"
    st = g.pool_stats()
    assert st.ntotal == o.ntotal and st.blocks_in_use == o.blocks_in_use
    rng = np.random.default_rng(w.seed)
    order = np.argsort(sizes)
    lists = list(rng.choice(w.nlist, n_lists, replace=False)) + [int(order[-1]), int(order[-2]), int(order[0])]
    say(request, f"{w.name}: every list has the oracle's length; longest {int(sizes.max())} vectors, "
                 f"{st.blocks_in_use} blocks; comparing {len(lists)} lists bit for bit")
    compare_lists(g, o, lists, w.name)
    return sizes


def check_queries(request, w, g, o, q, batch, what):
    s = torch.cuda.Stream()
    got = {}
    for mode in scan_modes(g):  # dot products on the matrix cores, then on the vector unit
        got_d, got_i = [], []
        for lo in range(0, len(q), batch):
            d, i = g.search(dev(q[lo:lo + batch]), w.k, w.nprobe, stream=s)
            s.synchronize()
            got_d.append(d.cpu().numpy()); got_i.append(i.cpu().numpy())
        assert g.poll_error() == 0
        got[mode] = (np.concatenate(got_d), np.concatenate(got_i))
    probes = g.probe(dev(q[:batch]), w.nprobe).cpu().numpy()
    assert np.array_equal(probes, o.probe(q[:batch], w.nprobe)), f"{what}: probed lists differ"
    say(request, f"{what}: {len(q)} queries answered on the GPU; the oracle's turn")
    rd, ri = o.search(q, w.k, w.nprobe)
    for mode, (gd, gi) in got.items():
        assert_topk_matches(w.metric, gd, gi, rd, ri, rtol=RTOL, atol=ATOL, what=f"{what}, scan_mfma {mode}")


