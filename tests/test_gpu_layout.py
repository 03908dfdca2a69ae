"""The pool's bytes, read without the library: the caller owns the pool tensor, so a test can take a
list apart by the documented layout alone (block stride and offset of the first block from
rtams_pool_stats, the chain from rtams_list_chain) and compare with the oracle.  Block = header of 128
bytes (int32 prev, next, owner, seq, capacity, size), T_m int64 ids, then the vectors in groups of 64:
inside a group the float4 of dimensions 4c..4c+3 of vector v lies at float4 index (c * 64 + v), i.e.
float index ((group * d/4 + c) * 64 + v) * 4 + j (the paper's interleaved layout, its equation for
"mv", re-derived for 64-wide wavefronts).  A layout that differed from this one but agreed with itself
(fill, scan and export all go through one index function) would pass every other test."""
import numpy as np
import pytest
import torch

from paper_2408_02937_amd import synth
from tests.gpu_common import dev, make_pair

pytestmark = pytest.mark.gpu

HEADER_BYTES = 128


def list_from_raw_bytes(pool: np.ndarray, first_block_at: int, stride: int, chain, T_m: int, d: int, length: int):
    ids, vecs = [], []
    for seq, b in enumerate(chain):
        at = first_block_at + int(b) * stride
        prev, nxt, owner, bseq, capacity, size = pool[at:at + 24].view(np.int32)
        want = min(T_m, length - seq * T_m)
        assert (capacity, size, bseq) == (T_m, want, seq), f"block {b}: header says capacity {capacity} size {size} seq {bseq}"
        assert prev == (chain[seq - 1] if seq else -1) and nxt == (chain[seq + 1] if seq + 1 < len(chain) else -1)
        ids.append(pool[at + HEADER_BYTES:at + HEADER_BYTES + 8 * T_m].view(np.int64)[:want].copy())
        raw = pool[at + HEADER_BYTES + 8 * T_m:at + HEADER_BYTES + 8 * T_m + 4 * T_m * d].view(np.float32)
        x = raw.reshape(T_m // 64, d // 4, 64, 4).transpose(0, 2, 1, 3).reshape(T_m, d)  # group, vector, chunk, j
        vecs.append(x[:want].copy())
        yield_owner = owner
    return np.concatenate(ids), np.concatenate(vecs), yield_owner


@pytest.mark.parametrize("name", ["byte-l2", "unit-ip"])
def test_lists_can_be_read_from_the_pool_bytes_by_the_documented_layout(name):
    if name == "byte-l2":
        w = synth.byte_valued_l2("layout-byte", 61, n_base=20_000, n_centres=40, nlist=48, block_vecs=128,
                                 n_queries=8, n_inserts=2_000, insert_batch=64, nprobe=4, k=10)
    else:
        w = synth.unit_ip("layout-ip", 62, d=96, n_base=20_000, n_centres=300, nlist=64, block_vecs=256,
                          n_queries=8, n_inserts=2_048, insert_batch=512, nprobe=4, k=10)
    print(f"[case] {w.name} seed={w.seed}", flush=True)
    g, o = make_pair(w)
    g.set_param("ordered_add", 1)  # positions in the order of the batch: the oracle's sequences, entry by entry
    g.add(dev(w.base)); o.add(w.base)
    for b in range(0, len(w.inserts), w.insert_batch):
        g.add(dev(w.inserts[b:b + w.insert_batch])); o.add(w.inserts[b:b + w.insert_batch])
    g.rearrange(int(np.argmax(g.list_sizes()))); o.rearrange(int(np.argmax(o.list_sizes())))  # moved blocks too
    torch.cuda.synchronize()
    st = g.pool_stats()
    pool = g.pool.cpu().numpy()
    sizes = g.list_sizes()
    for k in range(w.nlist):
        chain = g.list_chain(k)
        assert len(chain) == (sizes[k] + w.block_vecs - 1) // w.block_vecs
        if sizes[k] == 0:
            continue
        ids, x, owner = list_from_raw_bytes(pool, st.meta_bytes, st.block_bytes, chain, w.block_vecs, w.d, int(sizes[k]))
        assert owner == k
        oi, ox = o.list_export(k)
        assert np.array_equal(ids, oi), f"list {k}: ids read from the pool differ from the oracle's sequence"
        assert np.array_equal(x.view(np.uint32), ox.view(np.uint32)), f"list {k}: vectors read from the pool differ"
    g.close()
