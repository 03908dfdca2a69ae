"""ctypes front end of the CPU oracle (rtams_oracle.c).

TEST INFRASTRUCTURE: imported only by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing here touches the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rtams_oracle.c")
_LIB = os.path.join(_HERE, "librtams_oracle.so")

L2, IP = 0, 1
STORAGE = {"f32": 0, "f16": 1, "u8": 2}
OK, EINVAL, ESTATE, EPOOL = 0, -1, -2, -3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps every multiply and
    add as written; fma() calls become the hardware instruction (-mfma)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-mfma", "-shared",
               "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
        L.orc_create.restype = vp
        L.orc_create.argtypes = [i32, i32, i32, i64, i64, i64]
        L.orc_destroy.argtypes = [vp]
        L.orc_set_centroids.argtypes = [vp, vp]
        L.orc_set_codebooks.argtypes = [vp, i32, vp]
        L.orc_set_storage.argtypes = [vp, i32]
        L.orc_stored.restype = None
        L.orc_stored.argtypes = [i32, i64, vp, vp]
        L.orc_pq_encode.argtypes = [vp, i64, vp, vp]
        L.orc_list_export_codes.argtypes = [vp, i32, vp, vp]
        L.orc_assign.argtypes = [vp, i64, vp, vp]
        L.orc_coarse_scores.argtypes = [vp, vp, vp]
        L.orc_add.argtypes = [vp, i64, vp, vp, vp]
        L.orc_rearrange.argtypes = [vp, i32]
        L.orc_probe.argtypes = [vp, i64, vp, i32, vp]
        L.orc_search.argtypes = [vp, i64, vp, i32, i32, vp, vp]
        for name in ("orc_ntotal", "orc_blocks_in_use", "orc_cur_P", "orc_nfree", "orc_n_rearrange"):
            getattr(L, name).restype = i64
            getattr(L, name).argtypes = [vp]
        for name in ("orc_list_size", "orc_list_blocks", "orc_list_online", "orc_list_jumps"):
            getattr(L, name).restype = i64
            getattr(L, name).argtypes = [vp, i32]
        L.orc_list_export.argtypes = [vp, i32, vp, vp]
        L.orc_list_chain.argtypes = [vp, i32, vp]
        L.orc_slot.argtypes = [vp, i32, i64, vp, vp]
        L.orc_pool_bytes_in_use.restype = i64
        L.orc_pool_bytes_in_use.argtypes = [vp, i64]
        L.orc_threads.restype = i32
        _lib = L
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"oracle {what}: error {code}")
        self.code = code


class OracleIndex:
    """Block-based inverted-list index, sequential reference semantics."""

    def __init__(self, d: int, nlist: int, metric: str = "l2", block_vecs: int = 64,
                 rearrange_threshold: int = 0, pool_blocks: int = 1 << 20):
        self.d, self.nlist, self.block_vecs = d, nlist, block_vecs
        self.metric = {"l2": L2, "ip": IP}[metric]
        self._h = lib().orc_create(d, nlist, self.metric, block_vecs, rearrange_threshold, pool_blocks)
        if not self._h:
            raise OracleError(EINVAL, "create")

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_destroy(self._h)
            self._h = None

    def _chk(self, rc: int, what: str):
        if rc != OK:
            raise OracleError(rc, what)

    def set_centroids(self, centroids) -> None:
        c = _f32(centroids)
        assert c.shape == (self.nlist, self.d)
        self._chk(lib().orc_set_centroids(self._h, _ptr(c)), "set_centroids")

    def set_storage(self, storage: str) -> None:
        """What flat lists keep of a vector: "f32", "f16" or "u8" (before the first add)."""
        self._chk(lib().orc_set_storage(self._h, STORAGE[storage]), "set_storage")

    def set_codebooks(self, codebooks) -> None:
        """codebooks [M][256][d / M]: the lists hold product-quantiser codes from here on."""
        cb = _f32(codebooks)
        m = cb.shape[0]
        assert cb.shape == (m, 256, self.d // m) and self.d % m == 0
        self.pq_m = m
        self._chk(lib().orc_set_codebooks(self._h, m, _ptr(cb)), "set_codebooks")

    def pq_encode(self, vecs) -> np.ndarray:
        y = _f32(vecs).reshape(-1, self.d)
        out = np.empty((y.shape[0], self.pq_m), dtype=np.uint8)
        self._chk(lib().orc_pq_encode(self._h, y.shape[0], _ptr(y), _ptr(out)), "pq_encode")
        return out

    def list_export_codes(self, k: int) -> Tuple[np.ndarray, np.ndarray]:
        n = self.list_size(k)
        ids = np.empty(n, dtype=np.int64)
        codes = np.empty((n, self.pq_m), dtype=np.uint8)
        lib().orc_list_export_codes(self._h, k, _ptr(ids), _ptr(codes))
        return ids, codes

    def assign(self, vecs) -> np.ndarray:
        y = _f32(vecs)
        out = np.empty(y.shape[0], dtype=np.int32)
        self._chk(lib().orc_assign(self._h, y.shape[0], _ptr(y), _ptr(out)), "assign")
        return out

    def coarse_scores(self, vec) -> np.ndarray:
        y = _f32(vec).reshape(self.d)
        out = np.empty(self.nlist, dtype=np.float64)
        self._chk(lib().orc_coarse_scores(self._h, _ptr(y), _ptr(out)), "coarse_scores")
        return out

    def add(self, vecs, ids=None, assign=None) -> None:
        """Inserts the vectors one after the other.  `assign` may carry the list of each vector as
        assign() would compute it (a parallel pass done beforehand, or an assignment known and
        checked by other means); None computes it here."""
        y = _f32(vecs).reshape(-1, self.d)
        i = None if ids is None else np.ascontiguousarray(ids, dtype=np.int64)
        a = None if assign is None else np.ascontiguousarray(assign, dtype=np.int32)
        assert a is None or a.shape == (y.shape[0],)
        self._chk(lib().orc_add(self._h, y.shape[0], _ptr(y), _ptr(i), _ptr(a)), "add")

    def rearrange(self, lst: int) -> None:
        self._chk(lib().orc_rearrange(self._h, lst), "rearrange")

    def probe(self, queries, nprobe: int) -> np.ndarray:
        q = _f32(queries).reshape(-1, self.d)
        out = np.empty((q.shape[0], nprobe), dtype=np.int32)
        self._chk(lib().orc_probe(self._h, q.shape[0], _ptr(q), nprobe, _ptr(out)), "probe")
        return out

    def search(self, queries, k: int, nprobe: int) -> Tuple[np.ndarray, np.ndarray]:
        q = _f32(queries).reshape(-1, self.d)
        dist = np.empty((q.shape[0], k), dtype=np.float64)
        ids = np.empty((q.shape[0], k), dtype=np.int64)
        self._chk(lib().orc_search(self._h, q.shape[0], _ptr(q), k, nprobe, _ptr(dist), _ptr(ids)),
                  "search")
        return dist, ids

    # introspection
    @property
    def ntotal(self) -> int:
        return lib().orc_ntotal(self._h)

    @property
    def blocks_in_use(self) -> int:
        return lib().orc_blocks_in_use(self._h)

    @property
    def cur_P(self) -> int:
        return lib().orc_cur_P(self._h)

    @property
    def nfree(self) -> int:
        return lib().orc_nfree(self._h)

    @property
    def n_rearrange(self) -> int:
        return lib().orc_n_rearrange(self._h)

    def list_size(self, k: int) -> int:
        return lib().orc_list_size(self._h, k)

    def list_sizes(self) -> np.ndarray:
        return np.array([self.list_size(k) for k in range(self.nlist)], dtype=np.int64)

    def list_blocks(self, k: int) -> int:
        return lib().orc_list_blocks(self._h, k)

    def list_online(self, k: int) -> int:
        return lib().orc_list_online(self._h, k)

    def list_jumps(self, k: int) -> int:
        return lib().orc_list_jumps(self._h, k)

    def list_export(self, k: int) -> Tuple[np.ndarray, np.ndarray]:
        n = self.list_size(k)
        ids = np.empty(n, dtype=np.int64)
        x = np.empty((n, self.d), dtype=np.float32)
        lib().orc_list_export(self._h, k, _ptr(ids), _ptr(x))
        return ids, x

    def list_chain(self, k: int) -> np.ndarray:
        ch = np.empty(self.list_blocks(k), dtype=np.int32)
        lib().orc_list_chain(self._h, k, _ptr(ch))
        return ch

    def slot(self, k: int, did: int) -> Tuple[int, int]:
        b, o = C.c_int32(), C.c_int64()
        lib().orc_slot(self._h, k, did, C.byref(b), C.byref(o))
        return b.value, o.value

    def pool_bytes_in_use(self, header_bytes: int = 0) -> int:
        return lib().orc_pool_bytes_in_use(self._h, header_bytes)


def stored(storage: str, values) -> np.ndarray:
    """What a list with this storage keeps of each value (float32 in, float32 out)."""
    v = _f32(values)
    out = np.empty_like(v)
    lib().orc_stored(STORAGE[storage], v.size, _ptr(v), _ptr(out))
    return out


def threads() -> int:
    return lib().orc_threads()
