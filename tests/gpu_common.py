"""Helpers of the GPU parity tests: build the HIP index and the oracle from the
same workload, compare list contents canonically."""
from __future__ import annotations

import numpy as np
import torch

from oracle.oracle import OracleIndex
from paper_2408_02937_amd import rtams


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def make_pair(w, pool_blocks=None, rearrange_threshold=0, max_batch=256, max_k=128, max_nprobe=64,
              candidates_per_query=None, n_resources=4, max_add_batch=65536):
    """(gpu index, oracle index) over workload w, centroids set, nothing added."""
    n_all = len(w.base) + len(w.inserts)
    if pool_blocks is None:
        pool_blocks = n_all // w.block_vecs + 2 * w.nlist + 8
    if candidates_per_query is None:
        candidates_per_query = n_all + 64
    g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=pool_blocks,
                    rearrange_threshold=rearrange_threshold, n_resources=n_resources,
                    max_batch=max_batch, max_k=max_k, max_nprobe=min(max_nprobe, w.nlist),
                    max_add_batch=max_add_batch, candidates_per_query=candidates_per_query)
    g.set_centroids(dev(w.centroids))
    o = OracleIndex(w.d, w.nlist, w.metric, w.block_vecs, rearrange_threshold=rearrange_threshold,
                    pool_blocks=pool_blocks)
    o.set_centroids(w.centroids)
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
