"""CPU-only checks of the HIP library's boundary: it loads, exports every symbol the
header declares, and its host-side argument checks work without a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2408_02937_amd import rtams

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    found = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):  # rtams.h and rtams_measure.h
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        found |= set(re.findall(r"\b(rtams_[a-z_]+)\s*\(", text))
    return sorted(found)


def test_library_exports_every_declared_symbol():
    L = rtams.lib()
    declared = header_symbols()
    assert declared == sorted(rtams.SYMBOLS)
    for name in declared:
        assert hasattr(L, name), name


def cfg(**kw):
    base = dict(d=32, nlist=64, metric=0, block_vecs=64, rearrange_threshold=0, n_resources=4,
                max_batch=16, max_k=10, max_nprobe=8, max_add_batch=1024)
    base.update(kw)
    return rtams.Config(**base)


def test_reserve_size_arithmetic():
    L = rtams.lib()
    f = L.rtams_overflow_bytes_for
    assert f(4, 1000) == 256 + 2 * 4 * 4096          # 4000 bytes round up to whole 256-byte units
    assert f(1, 64) == 256 + 2 * 256 and f(32, 0) == 256
    assert f(0, 10) == 0 and f(33, 10) == 0 and f(4, -1) == 0


def test_pool_size_arithmetic():
    L = rtams.lib()
    c = cfg()
    one = L.rtams_pool_bytes_for(C.byref(c), 1)
    many = L.rtams_pool_bytes_for(C.byref(c), 1001)
    stride = (many - one) // 1000
    # a block is header + T_m ids + T_m vectors, padded to 256 bytes, plus 16 bytes of tables
    payload = 128 + 64 * 8 + 64 * 32 * 4
    padded = (payload + 255) // 256 * 256
    assert abs(stride - (padded + 16)) <= 1          # alignment of the tables rounds the quotient
    # per candidate: key + position, should it survive the pruning bound
    assert L.rtams_scratch_bytes_for(C.byref(c), 1000) - L.rtams_scratch_bytes_for(C.byref(c), 0) \
        in range(16 * 1000 * 8, 16 * 1000 * 8 + 2 * 256 + 1)


@pytest.mark.parametrize("bad", [dict(d=30), dict(d=0), dict(block_vecs=100), dict(nlist=0), dict(metric=7),
                                 dict(max_k=2000), dict(max_nprobe=65), dict(n_resources=0)])
def test_bad_configurations_are_refused_on_the_host(bad):
    L = rtams.lib()
    c = cfg(**bad)
    assert L.rtams_pool_bytes_for(C.byref(c), 10) == 0
    h = C.c_void_p()
    assert L.rtams_create(C.byref(c), C.byref(h)) == rtams.EINVAL and not h.value
    assert len(L.rtams_last_error()) > 0


def test_create_needs_memory():
    L = rtams.lib()
    h = C.c_void_p()
    assert L.rtams_create(C.byref(cfg()), C.byref(h)) == rtams.EINVAL
    assert b"pool and scratch" in L.rtams_last_error()


def test_a_pool_of_more_than_2_to_32_places_is_refused_on_the_host():
    """A search names a surviving candidate by its place in the pool, a 32-bit number: create says
    EINVAL for a pool that would hold more places, and how many bytes it may have.  (The sizes are
    checked before any memory is touched: the addresses given here are never used.)"""
    L = rtams.lib()
    c = cfg(d=4, block_vecs=64)
    limit_blocks = (1 << 32) // 64
    fits = L.rtams_pool_bytes_for(C.byref(c), limit_blocks)
    c.d_pool, c.d_scratch = 0x10000, 0x20000
    c.scratch_bytes = 1 << 30
    c.pool_bytes = L.rtams_pool_bytes_for(C.byref(c), limit_blocks + 4096)
    assert c.pool_bytes > fits > 0
    h = C.c_void_p()
    assert L.rtams_create(C.byref(c), C.byref(h)) == rtams.EINVAL and not h.value
    msg = L.rtams_last_error().decode()
    assert "2^32 places" in msg and str(fits) in msg


@pytest.mark.parametrize("bad_m", [3, 6, 12, 68, -4])
def test_bad_quantiser_shapes_are_refused_on_the_host(bad_m):
    """pq_m must be 0, or a multiple of 4 up to 64 that divides d (here d = 32)."""
    L = rtams.lib()
    assert L.rtams_pool_bytes_for(C.byref(cfg(pq_m=bad_m)), 10) == 0
    assert b"pq_m" in L.rtams_last_error()


def test_quantised_blocks_are_smaller_and_carry_a_table_per_query():
    L = rtams.lib()
    flat, pq = cfg(), cfg(pq_m=8)
    stride = lambda c: (L.rtams_pool_bytes_for(C.byref(c), 2010) - L.rtams_pool_bytes_for(C.byref(c), 1010)) // 1000
    # header 128 + 64 ids + 64 x 8 code bytes = 1152 -> 1280 with the 256-byte padding, plus 16 bytes of tables
    assert abs(stride(pq) - (1280 + 16)) <= 1 and stride(pq) < stride(flat)
    # per query a table of pq_m x 256 floats in every stream resource
    extra = L.rtams_scratch_bytes_for(C.byref(pq), 0) - L.rtams_scratch_bytes_for(C.byref(flat), 0)
    assert extra == 16 * 8 * 256 * 4


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.parametrize("bad", [dict(storage=3), dict(storage=-1), dict(storage=1, d=36), dict(storage=2, d=40),
                                 dict(storage=1, pq_m=8), dict(storage=2, pq_m=8)])
def test_bad_storage_is_refused_on_the_host(bad):
    """Halves need d % 8 == 0, bytes d % 16 == 0, and quantised lists keep codes, not vectors."""
    L = rtams.lib()
    assert L.rtams_pool_bytes_for(C.byref(cfg(**bad)), 10) == 0
    assert b"storage" in L.rtams_last_error()


def test_narrow_storage_shrinks_the_blocks():
    L = rtams.lib()
    stride = lambda c: (L.rtams_pool_bytes_for(C.byref(c), 2010) - L.rtams_pool_bytes_for(C.byref(c), 1010)) // 1000
    f32, f16, u8 = (stride(cfg(storage=s)) for s in (0, 1, 2))
    # header 128 + 64 ids x 8 + 64 vectors x 32 dimensions x {4, 2, 1} bytes, padded to 256, plus 16 bytes of tables
    assert (f32, f16, u8) == (8960 + 16, 4864 + 16, 2816 + 16)    # 8832, 4736, 2688 padded
