"""Flat lists that keep half-precision numbers or bytes: HIP path against the
CPU oracle through the C ABI.  What a list keeps must be the oracle's
conversion bit for bit; scores are fp32 arithmetic on the converted vectors."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from paper_2408_02937_amd import rtams, synth
from tests.gpu_common import assert_lists_equal, dev, make_pair
from tests.helpers import assert_topk_matches, RTOL

pytestmark = pytest.mark.gpu



def cases():
    byte = synth.byte_valued_l2("st-byte", 51, n_base=30_000, n_centres=40, nlist=96, block_vecs=128, n_queries=300,
                                n_inserts=3_000, insert_batch=64, nprobe=12, k=100)
    rng = np.random.default_rng(52)
    frac = replace(byte, name="st-frac",  # the same with fractional parts and values past both ends of a byte
                   base=(byte.base * 1.05 - 6 + rng.uniform(-0.5, 0.5, byte.base.shape)).astype(np.float32),
                   inserts=(byte.inserts + rng.uniform(-0.5, 0.5, byte.inserts.shape)).astype(np.float32))
    out = {
        "f16-tiny-l2": ("f16", synth.config(1)),
        "f16-unit-ip": ("f16", synth.unit_ip("st-ip", 53, d=96, n_base=40_000, n_centres=300, nlist=128,
                                              block_vecs=256, n_queries=300, n_inserts=2_048, insert_batch=512,
                                              nprobe=16, k=10)),
        "f16-zipf-l2": ("f16", synth.skewed_l2("st-zipf", 54, d=72, n_base=60_000, nlist=256, block_vecs=64,
                                               n_queries=256, n_inserts=4_096, insert_batch=1024, nprobe=16, k=50)),
        "u8-byte-l2": ("u8", byte),
        "u8-byte-ip": ("u8", replace(synth.byte_valued_l2("st-byte-ip", 55, d=48, n_base=20_000, n_centres=30,
                                                          nlist=64, block_vecs=64, n_queries=200, n_inserts=1_000,
                                                          insert_batch=100, nprobe=8, k=20), metric="ip")),
        "u8-fractional-l2": ("u8", frac),
        # 15,000 candidates per query: the pruning bound and its sample over byte chunks are at work
        "u8-dense-l2": ("u8", synth.byte_valued_l2("st-dense", 56, d=64, n_base=60_000, n_centres=30, nlist=64,
                                                   block_vecs=128, n_queries=300, n_inserts=640, insert_batch=64,
                                                   nprobe=16, k=100)),
        "f16-dense-ip": ("f16", synth.unit_ip("st-dense-ip", 57, d=64, n_base=60_000, n_centres=100, nlist=64,
                                              block_vecs=128, n_queries=300, n_inserts=512, insert_batch=512,
                                              nprobe=16, k=20)),
    }
    return out


@pytest.fixture(scope="module", params=list(cases().keys()))
def loaded(request):
    storage, w = cases()[request.param]
    print(f"[case] storage={storage} workload={w.name} metric={w.metric} d={w.d}", flush=True)
    g, o = make_pair(w, storage=storage)
    g.set_param("use_mfma", 2)
    g.add(dev(w.base)); o.add(w.base)
    bounds = [len(w.base)]
    for b in range(0, len(w.inserts), w.insert_batch):
        chunk = w.inserts[b:b + w.insert_batch]
        g.add(dev(chunk)); o.add(chunk)
        bounds.append(bounds[-1] + len(chunk))
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    yield storage, w, g, o, np.array(bounds[:-1])
    g.close()


def test_lists_keep_the_oracle_s_conversion_bit_for_bit(loaded):
    storage, w, g, o, bounds = loaded
    g.validate()
    assert_lists_equal(g, o, bounds)       # exported vectors are the converted ones on both sides
    changed = sum(int((o.list_export(k)[1] != 0).any()) for k in range(4))
    assert changed > 0


@pytest.mark.parametrize("batch", [1, 7, 64, 256])
def test_search_matches_the_oracle(loaded, batch):
    storage, w, g, o, _ = loaded
    q = w.queries[:batch]
    d, i = g.search(dev(q), w.k, w.nprobe)
    torch.cuda.synchronize()
    assert g.poll_error() == 0
    rd, ri = o.search(q, w.k, w.nprobe)
    assert_topk_matches(w.metric, d.cpu().numpy(), i.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6,
                        what=f"{storage} {w.name} batch {batch}")


def test_byte_storage_of_byte_valued_data_answers_exactly_as_float_storage():
    w = cases()["u8-byte-l2"][1]
    print(f"[case] u8 against f32 storage, workload={w.name}", flush=True)
    (g8, o8), (g32, _) = make_pair(w, storage="u8"), make_pair(w)
    for g in (g8, g32):
        g.add(dev(w.base))
    o8.add(w.base)
    q = dev(w.queries[:256])
    (d8, i8), (d32, i32) = g8.search(q, w.k, w.nprobe), g32.search(q, w.k, w.nprobe)
    torch.cuda.synchronize()
    assert torch.equal(d8, d32) and torch.equal(i8, i32)
    rd, ri = o8.search(w.queries[:256], w.k, w.nprobe)
    assert np.array_equal(d8.cpu().numpy().astype(np.float64), rd) and np.array_equal(i8.cpu().numpy(), ri)
    # a quarter of the bytes per block
    assert g8.pool_stats().block_bytes < g32.pool_stats().block_bytes / 3
    g8.close(); g32.close()


@pytest.mark.parametrize("storage", ["f16", "u8"])
def test_rearrangement_moves_narrow_blocks_whole(storage):
    rng = np.random.default_rng(7)
    d, T, nlist = 32, 64, 3
    C = (np.eye(nlist, d) * 100 + 60).astype(np.float32)
    w = synth.Workload("st-interleaved", "l2", d, nlist, T, nlist, 10, np.zeros((0, d), np.float32), C,
                       np.zeros((0, d), np.float32), np.zeros((0, d), np.float32), 1, 7)
    print(f"[case] rearrangement with storage={storage}", flush=True)
    g, o = make_pair(w, pool_blocks=100, candidates_per_query=8192, storage=storage)
    for r in range(5):
        for k in range(nlist):
            y = (C[k] + 3.0 * rng.standard_normal((T, d))).astype(np.float32)
            g.add(dev(y)); o.add(y)
    g.rearrange(1)
    torch.cuda.synchronize()
    g.validate()
    assert g.list_info(1)[1] == 1
    assert_lists_equal(g, o)
    q = (C[1] + rng.standard_normal((8, d))).astype(np.float32)
    dd, ii = g.search(dev(q), 10, 3)
    torch.cuda.synchronize()
    rd, ri = o.search(q, 10, 3)
    assert_topk_matches("l2", dd.cpu().numpy(), ii.cpu().numpy(), rd, ri, rtol=RTOL, atol=1e-6)
    g.close()


@pytest.mark.parametrize("storage", ["f16", "u8"])
def test_conversion_of_edge_values(storage):
    """Ties, the ends of the range, subnormal halves, signed zeros, not-a-number (bytes): what
    the fill kernel writes is what the oracle's conversion gives, read back through the export."""
    from oracle import oracle
    print(f"[case] edge values, storage={storage}", flush=True)
    if storage == "f16":
        halves = np.arange(0, 0x7C00, 37, dtype=np.uint16).view(np.float16).astype(np.float64)
        nxt = (np.arange(0, 0x7C00, 37, dtype=np.uint16) + 1).view(np.float16).astype(np.float64)
        vals = np.concatenate([halves, (halves + nxt) / 2, -(halves + nxt) / 2,
                               [65504, 65519.996, 65520, 1e6, -65520, 2.0 ** -24, 1.5 * 2.0 ** -24, 2.5 * 2.0 ** -24,
                                2.0 ** -25, 2.0 ** -25 * 1.0001, 2.0 ** -26, 2.0 ** -14 - 2.0 ** -25, 0.0, -0.0, 0.1,
                                1 / 3]]).astype(np.float32)
    else:
        vals = np.concatenate([np.arange(-4, 520) / 2, [np.nan, -0.0, 254.5, 255.5, 1e9, -1e9, 127.49999, 0.49999997],
                               np.random.default_rng(3).uniform(-20, 280, 500)]).astype(np.float32)
    d = 16
    pad = (-len(vals)) % d
    x = np.concatenate([vals, np.zeros(pad, np.float32)]).reshape(-1, d)
    g = rtams.Index(d, 1, "ip", 64, pool_blocks=len(x) // 64 + 4, max_batch=8, max_k=8, max_nprobe=1,
                    candidates_per_query=4096, n_resources=1, storage=storage)
    g.set_centroids(dev(np.zeros((1, d), np.float32)))
    g.add(dev(x))
    torch.cuda.synchronize()
    ids, got = g.list_export(0)
    got = got.cpu().numpy()[np.argsort(ids.cpu().numpy())]
    want = oracle.stored(storage, x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    g.close()
