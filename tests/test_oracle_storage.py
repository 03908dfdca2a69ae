"""Pins of the oracle's narrow storage (half precision, bytes) against things
that are not the oracle: numpy's IEEE conversions, brute force over vectors
converted independently, and the flat index itself where nothing is lost."""
import numpy as np
import pytest

from oracle import oracle
from oracle.oracle import OracleIndex
from paper_2408_02937_amd import synth
from tests.helpers import assert_topk_matches, brute_force_topk


def numpy_half(x):
    with np.errstate(over="ignore"):
        return x.astype(np.float16).astype(np.float32)


def numpy_byte(x):
    r = np.clip(np.rint(np.nan_to_num(x, nan=0.0, posinf=255.0, neginf=0.0)), 0, 255).astype(np.float32)
    return r + np.float32(0.0)  # -0.0 -> +0.0 is not needed after clip: clip returns +0.0 for negatives


def test_half_conversion_is_ieee_round_to_nearest_even():
    rng = np.random.default_rng(5)
    parts = [
        # all magnitudes a half can hold, and beyond on both sides
        (rng.standard_normal(200_000) * np.exp2(rng.integers(-30, 18, 200_000))).astype(np.float32),
        # every half itself, and the exact midpoints between neighbouring halves (ties)
        np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float32),
        ((np.arange(0, 0x7BFF, dtype=np.uint16).view(np.float16).astype(np.float64)
          + np.arange(1, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)) / 2).astype(np.float32),
        # around the overflow threshold (65504 is the largest half, 65520 the first value that becomes infinity)
        np.array([65504, 65519.996, 65520, 65536, 1e6, -65519.996, -65520], dtype=np.float32),
        # subnormal halves: multiples of 2^-24, their midpoints, and what vanishes
        np.array([2.0 ** -24, 1.5 * 2.0 ** -24, 2.5 * 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001, 2.0 ** -26,
                  2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 0.0, -0.0, np.inf, -np.inf], dtype=np.float32),
    ]
    x = np.concatenate(parts + [-np.concatenate(parts[:3])])
    got, want = oracle.stored("f16", x), numpy_half(x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.isnan(oracle.stored("f16", np.array([np.nan], np.float32))[0])


def test_byte_conversion_rounds_to_even_and_clamps():
    rng = np.random.default_rng(6)
    x = np.concatenate([rng.uniform(-20, 280, 100_000).astype(np.float32),
                        np.arange(-4, 520, dtype=np.float32) / 2,          # every tie x.5
                        np.array([np.nan, np.inf, -np.inf, -0.0, 254.5, 255.5, 1e9], np.float32)])
    got = oracle.stored("u8", x)
    assert np.array_equal(got, numpy_byte(x)) and not np.signbit(got).any()
    b = np.arange(256, dtype=np.float32)
    assert np.array_equal(oracle.stored("u8", b), b)                     # byte values are kept as they are
    assert oracle.stored("u8", np.array([0.5, 1.5, 2.5], np.float32)).tolist() == [0.0, 2.0, 2.0]


@pytest.mark.parametrize("storage,metric", [("f16", "l2"), ("f16", "ip"), ("u8", "l2")])
def test_lists_hold_the_converted_vectors_of_the_flat_index_and_search_is_brute_force_on_them(storage, metric):
    if storage == "u8":
        w = synth.byte_valued_l2("t", 8, d=32, n_base=3000, n_centres=20, nlist=16, block_vecs=64, n_queries=30,
                                 n_inserts=10)
        base = (w.base + np.random.default_rng(1).uniform(-0.49, 0.49, w.base.shape)).astype(np.float32)
    else:
        w = (synth.gaussian_l2 if metric == "l2" else synth.unit_ip)("t", 8, d=24, n_base=3000, n_centres=20,
                                                                    nlist=16, block_vecs=64, n_queries=30, n_inserts=10)
        base = w.base
    flat = OracleIndex(w.d, w.nlist, metric, 64); flat.set_centroids(w.centroids); flat.add(base)
    ix = OracleIndex(w.d, w.nlist, metric, 64); ix.set_centroids(w.centroids); ix.set_storage(storage); ix.add(base)
    convert = numpy_half if storage == "f16" else numpy_byte
    # membership is decided by the vector as given; the list keeps the conversion
    assert np.array_equal(ix.list_sizes(), flat.list_sizes())
    changed = 0
    for k in range(w.nlist):
        (ia, xa), (ib, xb) = ix.list_export(k), flat.list_export(k)
        assert np.array_equal(ia, ib) and np.array_equal(xa.view(np.uint32), convert(xb).view(np.uint32))
        changed += int((xa != xb).sum())
        assert ix.list_blocks(k) == flat.list_blocks(k)
    assert changed > 0
    # every list probed: exhaustive search over the converted vectors
    conv, ids = convert(base), np.arange(len(base), dtype=np.int64)
    d, i = ix.search(w.queries, 10, w.nlist)
    for r in range(len(w.queries)):
        bd, bi = brute_force_topk(metric, conv, ids, w.queries[r], 10)
        assert_topk_matches(metric, d[r:r + 1], i[r:r + 1], bd[None], bi[None], rtol=1e-12)


def test_byte_storage_loses_nothing_on_byte_valued_data():
    w = synth.byte_valued_l2("t", 9, d=32, n_base=3000, n_centres=20, nlist=16, block_vecs=64, n_queries=30,
                             n_inserts=10)
    flat = OracleIndex(w.d, w.nlist, "l2", 64); flat.set_centroids(w.centroids); flat.add(w.base)
    ix = OracleIndex(w.d, w.nlist, "l2", 64); ix.set_centroids(w.centroids); ix.set_storage("u8"); ix.add(w.base)
    (d1, i1), (d2, i2) = flat.search(w.queries, 50, 4), ix.search(w.queries, 50, 4)
    assert np.array_equal(d1, d2) and np.array_equal(i1, i2)


def test_storage_is_fixed_before_the_first_vector_and_excludes_codebooks():
    from oracle.oracle import OracleError
    ix = OracleIndex(4, 2, "l2", 4); ix.set_centroids(np.eye(2, 4, dtype=np.float32))
    ix.set_storage("f16"); ix.set_storage("f32")
    ix.add(np.zeros((1, 4), np.float32))
    with pytest.raises(OracleError):
        ix.set_storage("u8")
    jx = OracleIndex(4, 2, "l2", 4); jx.set_centroids(np.eye(2, 4, dtype=np.float32)); jx.set_storage("u8")
    with pytest.raises(OracleError):
        jx.set_codebooks(np.zeros((2, 256, 2), np.float32))
