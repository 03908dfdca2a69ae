"""Thin Python binding of librtams.so: the same calls as include/rtams.h.

Argument marshalling only.  PyTorch provides device memory (the caller-owned
pool and scratch, inputs, outputs) and streams; every step of the path runs in
the HIP kernels behind the C ABI.  There is no fallback: if the library is
missing or an entry point fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librtams.so")

L2, IP = 0, 1
OK, EINVAL, ESTATE, EPOOL, EBUSY, EHIP, ESCRATCH, ENOSPARE = 0, -1, -2, -3, -4, -5, -6, -7
STORAGE = {"f32": 0, "f16": 1, "u8": 2}  # what flat lists keep of a coordinate
_NAMES = {EINVAL: "EINVAL", ESTATE: "ESTATE", EPOOL: "EPOOL", EBUSY: "EBUSY", EHIP: "EHIP",
          ESCRATCH: "ESCRATCH", ENOSPARE: "ENOSPARE"}

# every symbol include/rtams.h and include/rtams_measure.h declare
SYMBOLS = [
    "rtams_pool_bytes_for", "rtams_scratch_bytes_for", "rtams_create", "rtams_destroy",
    "rtams_set_centroids", "rtams_add", "rtams_search", "rtams_rearrange", "rtams_ntotal",
    "rtams_list_size", "rtams_list_info", "rtams_list_export", "rtams_list_chain",
    "rtams_list_sizes", "rtams_pool_stats", "rtams_validate", "rtams_probe", "rtams_assign",
    "rtams_poll_error", "rtams_clear_error", "rtams_last_error", "rtams_set_param", "rtams_scan_time",
    "rtams_copy_plain", "rtams_read_plain", "rtams_set_codebooks", "rtams_list_export_codes",
    "rtams_search_noalloc", "rtams_overflow_bytes_for", "rtams_scan_kernels",
]


class Config(C.Structure):
    _fields_ = [("d", C.c_int32), ("nlist", C.c_int32), ("metric", C.c_int32),
                ("block_vecs", C.c_int32), ("rearrange_threshold", C.c_int64),
                ("d_pool", C.c_void_p), ("pool_bytes", C.c_size_t),
                ("d_scratch", C.c_void_p), ("scratch_bytes", C.c_size_t),
                ("n_resources", C.c_int32), ("max_batch", C.c_int32), ("max_k", C.c_int32),
                ("max_nprobe", C.c_int32), ("max_add_batch", C.c_int32), ("pq_m", C.c_int32),
                ("storage", C.c_int32), ("overflow_bytes", C.c_size_t), ("overflow_chunks", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [("ntotal", C.c_int64), ("blocks_total", C.c_int64),
                ("blocks_handed_out", C.c_int64), ("blocks_free", C.c_int64),
                ("blocks_in_use", C.c_int64), ("block_bytes", C.c_int64),
                ("pool_bytes", C.c_int64), ("meta_bytes", C.c_int64), ("utilisation", C.c_double),
                ("lists_exceeding", C.c_int64), ("table_entries_used", C.c_int64),
                ("table_entries_total", C.c_int64), ("overflow_chunks", C.c_int64),
                ("overflow_chunk_entries", C.c_int64), ("overflow_chunks_leased", C.c_int64),
                ("rearrangement_state", C.c_int64), ("add_waits", C.c_int64)]


class RtamsError(RuntimeError):
    def __init__(self, code: int, what: str, detail: str):
        super().__init__(f"{what}: {_NAMES.get(code, code)}: {detail}")
        self.code = code


_lib = None


def lib():
    """Loads librtams.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` (build()) first")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        cp = C.POINTER(Config)
        L.rtams_pool_bytes_for.restype = C.c_size_t
        L.rtams_pool_bytes_for.argtypes = [cp, i64]
        L.rtams_scratch_bytes_for.restype = C.c_size_t
        L.rtams_scratch_bytes_for.argtypes = [cp, i64]
        L.rtams_overflow_bytes_for.restype = C.c_size_t
        L.rtams_overflow_bytes_for.argtypes = [i32, i64]
        L.rtams_create.argtypes = [cp, C.POINTER(vp)]
        L.rtams_destroy.argtypes = [vp]
        L.rtams_set_centroids.argtypes = [vp, vp, vp]
        L.rtams_set_codebooks.argtypes = [vp, vp, vp]
        L.rtams_list_export_codes.argtypes = [vp, i32, i64, vp, vp, C.POINTER(i64), vp]
        L.rtams_add.argtypes = [vp, i64, vp, vp, vp]
        L.rtams_search.argtypes = [vp, i64, vp, i32, i32, vp, vp, vp]
        L.rtams_search_noalloc.argtypes = [vp, i64, vp, i32, i32, vp, vp, vp]
        L.rtams_rearrange.argtypes = [vp, i32, vp]
        L.rtams_ntotal.argtypes = [vp, C.POINTER(i64)]
        L.rtams_list_size.argtypes = [vp, i32, C.POINTER(i64)]
        L.rtams_list_info.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
        L.rtams_list_export.argtypes = [vp, i32, i64, vp, vp, C.POINTER(i64), vp]
        L.rtams_list_chain.argtypes = [vp, i32, i64, vp, C.POINTER(i64)]
        L.rtams_list_sizes.argtypes = [vp, vp]
        L.rtams_pool_stats.argtypes = [vp, C.POINTER(Stats)]
        L.rtams_validate.argtypes = [vp, vp]
        L.rtams_probe.argtypes = [vp, i64, vp, i32, vp, vp]
        L.rtams_assign.argtypes = [vp, i64, vp, vp, vp]
        L.rtams_poll_error.argtypes = [vp]
        L.rtams_clear_error.argtypes = [vp]
        L.rtams_last_error.restype = C.c_char_p
        L.rtams_set_param.argtypes = [vp, C.c_char_p, i64]
        L.rtams_scan_time.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64), C.c_int]
        L.rtams_scan_kernels.argtypes = [vp, C.POINTER(i64), C.c_int]
        L.rtams_copy_plain.argtypes = [vp, vp, C.c_size_t, vp]
        L.rtams_read_plain.argtypes = [vp, C.c_size_t, vp, vp]
        _lib = L
    return _lib


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _chk(rc: int, what: str):
    if rc != OK:
        raise RtamsError(rc, what, lib().rtams_last_error().decode())


def _dev_f32(t: torch.Tensor, d: int, what: str) -> torch.Tensor:
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.dim() == 2 and t.shape[1] == d):
        raise ValueError(f"{what} must be a contiguous float32 CUDA tensor of shape [n][{d}]")
    return t


def copy_plain(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """The library's plain copy kernel (calibration of traffic counters)."""
    nbytes = src.numel() * src.element_size()
    _chk(lib().rtams_copy_plain(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream)), "rtams_copy_plain")


def read_plain(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """The library's plain read kernel (practical ceiling of a streaming read)."""
    nbytes = src.numel() * src.element_size()
    _chk(lib().rtams_read_plain(src.data_ptr(), nbytes, sink.data_ptr(), _stream_ptr(stream)), "rtams_read_plain")


class Index:
    """rtams_index over a pool and a scratch tensor that this object keeps alive."""

    def __init__(self, d: int, nlist: int, metric: str = "l2", block_vecs: int = 128,
                 pool_blocks: Optional[int] = None, pool_bytes: Optional[int] = None,
                 rearrange_threshold: int = 0, n_resources: int = 8, max_batch: int = 256,
                 max_k: int = 128, max_nprobe: int = 64, max_add_batch: int = 65536,
                 candidates_per_query: int = 65536, device: str = "cuda:0", pq_m: int = 0,
                 overflow_candidates: int = 0, overflow_chunks: int = 4, storage: str = "f32"):
        L = lib()
        self.d, self.nlist, self.block_vecs, self.pq_m = d, nlist, block_vecs, pq_m
        self.metric = {"l2": L2, "ip": IP}[metric]
        self.device = torch.device(device)
        cfg = Config(d=d, nlist=nlist, metric=self.metric, block_vecs=block_vecs,
                     rearrange_threshold=rearrange_threshold, n_resources=n_resources,
                     max_batch=max_batch, max_k=max_k, max_nprobe=min(max_nprobe, nlist),
                     max_add_batch=max_add_batch, pq_m=pq_m, storage=STORAGE[storage])
        self.storage = storage
        if pool_bytes is None:
            if pool_blocks is None:
                raise ValueError("give pool_blocks or pool_bytes")
            pool_bytes = L.rtams_pool_bytes_for(C.byref(cfg), pool_blocks)
            if pool_bytes == 0:
                raise RtamsError(EINVAL, "pool_bytes_for", L.rtams_last_error().decode())
        per_res = L.rtams_scratch_bytes_for(C.byref(cfg), candidates_per_query)
        if per_res == 0:
            raise RtamsError(EINVAL, "scratch_bytes_for", L.rtams_last_error().decode())
        # caller-owned device memory: one pool, one scratch area
        self.pool = torch.empty(pool_bytes, dtype=torch.uint8, device=self.device)
        # the reserve shared by all resources: overflow_chunks chunks of overflow_candidates entries
        overflow_bytes = 0
        if overflow_candidates > 0:
            overflow_bytes = L.rtams_overflow_bytes_for(overflow_chunks, overflow_candidates)
            if overflow_bytes == 0:
                raise RtamsError(EINVAL, "overflow_bytes_for", "overflow_chunks must be in 1..32")
        scratch_bytes = per_res * n_resources + overflow_bytes
        self.scratch = torch.empty(scratch_bytes, dtype=torch.uint8, device=self.device)
        cfg.d_pool, cfg.pool_bytes = self.pool.data_ptr(), pool_bytes
        cfg.d_scratch, cfg.scratch_bytes = self.scratch.data_ptr(), scratch_bytes
        cfg.overflow_bytes = overflow_bytes
        cfg.overflow_chunks = overflow_chunks
        self.cfg = cfg
        h = C.c_void_p()
        torch.cuda.synchronize(self.device)
        _chk(L.rtams_create(C.byref(cfg), C.byref(h)), "rtams_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib().rtams_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the path
    def set_centroids(self, centroids: torch.Tensor, stream=None) -> None:
        c = _dev_f32(centroids, self.d, "centroids")
        if c.shape[0] != self.nlist:
            raise ValueError("centroids must have nlist rows")
        _chk(lib().rtams_set_centroids(self._h, c.data_ptr(), _stream_ptr(stream)), "rtams_set_centroids")

    def set_codebooks(self, codebooks: torch.Tensor, stream=None) -> None:
        """codebooks [pq_m][256][d / pq_m] float32 on the device."""
        if (codebooks.dtype != torch.float32 or not codebooks.is_cuda or not codebooks.is_contiguous()
                or self.pq_m == 0 or tuple(codebooks.shape) != (self.pq_m, 256, self.d // self.pq_m)):
            raise ValueError("codebooks must be a contiguous float32 CUDA tensor [pq_m][256][d / pq_m]")
        _chk(lib().rtams_set_codebooks(self._h, codebooks.data_ptr(), _stream_ptr(stream)), "rtams_set_codebooks")

    def add(self, vecs: torch.Tensor, ids: Optional[torch.Tensor] = None, stream=None) -> None:
        v = _dev_f32(vecs, self.d, "vecs")
        ip = None
        if ids is not None:
            if not (ids.is_cuda and ids.dtype == torch.int64 and ids.is_contiguous() and ids.numel() == v.shape[0]):
                raise ValueError("ids must be a contiguous int64 CUDA tensor with one entry per vector")
            ip = ids.data_ptr()
        _chk(lib().rtams_add(self._h, v.shape[0], v.data_ptr(), ip, _stream_ptr(stream)), "rtams_add")

    def search(self, queries: torch.Tensor, k: int, nprobe: int, out_dist: Optional[torch.Tensor] = None,
               out_ids: Optional[torch.Tensor] = None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
        q = _dev_f32(queries, self.d, "queries")
        nq = q.shape[0]
        if out_dist is None:
            out_dist = torch.empty((nq, k), dtype=torch.float32, device=q.device)
        if out_ids is None:
            out_ids = torch.empty((nq, k), dtype=torch.int64, device=q.device)
        _chk(lib().rtams_search(self._h, nq, q.data_ptr(), k, nprobe, out_dist.data_ptr(),
                                out_ids.data_ptr(), _stream_ptr(stream)), "rtams_search")
        return out_dist, out_ids

    def search_noalloc(self, queries: torch.Tensor, k: int, nprobe: int, out_dist: torch.Tensor,
                       out_ids: torch.Tensor, stream=None) -> None:
        """rtams_search_noalloc: the request's scratch is the library's static array; the caller brings
        the output tensors ([nq][k] float32 and int64)."""
        q = _dev_f32(queries, self.d, "queries")
        nq = q.shape[0]
        if not (out_dist.is_cuda and out_dist.dtype == torch.float32 and out_dist.is_contiguous()
                and tuple(out_dist.shape) == (nq, k) and out_ids.is_cuda and out_ids.dtype == torch.int64
                and out_ids.is_contiguous() and tuple(out_ids.shape) == (nq, k)):
            raise ValueError("out_dist / out_ids must be contiguous CUDA tensors [nq][k] of float32 / int64")
        _chk(lib().rtams_search_noalloc(self._h, nq, q.data_ptr(), k, nprobe, out_dist.data_ptr(),
                                        out_ids.data_ptr(), _stream_ptr(stream)), "rtams_search_noalloc")

    def rearrange(self, lst: int = -1, stream=None) -> None:
        _chk(lib().rtams_rearrange(self._h, lst, _stream_ptr(stream)), "rtams_rearrange")

    # ---- introspection
    def probe(self, queries: torch.Tensor, nprobe: int, stream=None) -> torch.Tensor:
        q = _dev_f32(queries, self.d, "queries")
        out = torch.empty((q.shape[0], nprobe), dtype=torch.int32, device=q.device)
        _chk(lib().rtams_probe(self._h, q.shape[0], q.data_ptr(), nprobe, out.data_ptr(),
                               _stream_ptr(stream)), "rtams_probe")
        return out

    def assign(self, vecs: torch.Tensor, stream=None) -> torch.Tensor:
        v = _dev_f32(vecs, self.d, "vecs")
        out = torch.empty(v.shape[0], dtype=torch.int32, device=v.device)
        _chk(lib().rtams_assign(self._h, v.shape[0], v.data_ptr(), out.data_ptr(), _stream_ptr(stream)),
             "rtams_assign")
        return out

    @property
    def ntotal(self) -> int:
        v = C.c_int64()
        _chk(lib().rtams_ntotal(self._h, C.byref(v)), "rtams_ntotal")
        return v.value

    def list_size(self, lst: int) -> int:
        v = C.c_int64()
        _chk(lib().rtams_list_size(self._h, lst, C.byref(v)), "rtams_list_size")
        return v.value

    def list_sizes(self):
        import numpy as np
        out = np.empty(self.nlist, dtype=np.int64)
        _chk(lib().rtams_list_sizes(self._h, out.ctypes.data_as(C.c_void_p)), "rtams_list_sizes")
        return out

    def list_info(self, lst: int) -> Tuple[int, int, int]:
        b, r, o = C.c_int64(), C.c_int64(), C.c_int64()
        _chk(lib().rtams_list_info(self._h, lst, C.byref(b), C.byref(r), C.byref(o)), "rtams_list_info")
        return b.value, r.value, o.value

    def list_export(self, lst: int, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
        n = self.list_size(lst)
        ids = torch.empty(n, dtype=torch.int64, device=self.device)
        vecs = torch.empty((n, self.d), dtype=torch.float32, device=self.device)
        got = C.c_int64()
        _chk(lib().rtams_list_export(self._h, lst, n, ids.data_ptr(), vecs.data_ptr(), C.byref(got),
                                     _stream_ptr(stream)), "rtams_list_export")
        return ids[:got.value], vecs[:got.value]

    def list_export_codes(self, lst: int, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
        n = self.list_size(lst)
        ids = torch.empty(n, dtype=torch.int64, device=self.device)
        codes = torch.empty((n, max(self.pq_m, 1)), dtype=torch.uint8, device=self.device)
        got = C.c_int64()
        _chk(lib().rtams_list_export_codes(self._h, lst, n, ids.data_ptr(), codes.data_ptr(), C.byref(got),
                                           _stream_ptr(stream)), "rtams_list_export_codes")
        return ids[:got.value], codes[:got.value]

    def list_chain(self, lst: int):
        import numpy as np
        n = C.c_int64()
        rc = lib().rtams_list_chain(self._h, lst, 0, None, C.byref(n))
        if n.value == 0:
            _chk(rc, "rtams_list_chain")
            return np.empty(0, dtype=np.int32)
        out = np.empty(n.value, dtype=np.int32)
        _chk(lib().rtams_list_chain(self._h, lst, n.value, out.ctypes.data_as(C.c_void_p), C.byref(n)),
             "rtams_list_chain")
        return out

    def pool_stats(self) -> Stats:
        s = Stats()
        _chk(lib().rtams_pool_stats(self._h, C.byref(s)), "rtams_pool_stats")
        return s

    def validate(self, stream=None) -> None:
        _chk(lib().rtams_validate(self._h, _stream_ptr(stream)), "rtams_validate")

    def poll_error(self) -> int:
        return lib().rtams_poll_error(self._h)

    def clear_error(self) -> None:
        _chk(lib().rtams_clear_error(self._h), "rtams_clear_error")

    def scan_time(self, reset: bool = False) -> Tuple[float, int]:
        ms, n = C.c_double(), C.c_int64()
        _chk(lib().rtams_scan_time(self._h, C.byref(ms), C.byref(n), int(reset)), "rtams_scan_time")
        return ms.value, n.value

    def scan_kernels(self, reset: bool = False) -> dict:
        n = (C.c_int64 * 3)()
        _chk(lib().rtams_scan_kernels(self._h, n, int(reset)), "rtams_scan_kernels")
        return {"k_scan": n[0], "k_scan_mm": n[1], "k_pq_scan": n[2]}

    def set_param(self, key: str, value: int) -> None:
        _chk(lib().rtams_set_param(self._h, key.encode(), value), "rtams_set_param")
