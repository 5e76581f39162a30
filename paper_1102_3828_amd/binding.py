"""Thin ctypes binding of libivfadcr (include/ivfadcr.h): argument marshalling only.

Every step of index construction and search runs in the HIP library; PyTorch supplies
device memory and streams for the caller's buffers.  There is no CPU fallback: if the
library is not built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch  # noqa: F401  -- must be loaded first: the library binds to the HIP runtime that PyTorch ships, so
#                              that device pointers of torch tensors are valid inside it (one runtime per process)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libivfadcr.so")

OK, ERR_INVALID_ARG, ERR_STATE, ERR_OOM, ERR_HIP = 0, -1, -2, -3, -4


class IvfrError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"ivfadcr error {code}: {message}")
        self.code = code


class Params(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("c", ctypes.c_int32), ("m", ctypes.c_int32),
                ("m_refine", ctypes.c_int32), ("device", ctypes.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_1102_3828_amd.build` "
                          "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64
    sig = {
        "ivfr_create": (ctypes.c_int, [ctypes.POINTER(Params), ctypes.POINTER(vp)]),
        "ivfr_destroy": (ctypes.c_int, [vp]),
        "ivfr_train": (ctypes.c_int, [vp, vp, i64, i32, u64]),
        "ivfr_set_codebooks": (ctypes.c_int, [vp, vp, vp, vp]),
        "ivfr_get_codebooks": (ctypes.c_int, [vp, vp, vp, vp]),
        "ivfr_add": (ctypes.c_int, [vp, vp, i64, i64]),
        "ivfr_finalize": (ctypes.c_int, [vp]),
        "ivfr_ntotal": (i64, [vp]),
        "ivfr_export": (ctypes.c_int, [vp, vp, vp, vp, vp]),
        "ivfr_import": (ctypes.c_int, [vp, i64, vp, vp, vp, vp]),
        "ivfr_search": (ctypes.c_int, [vp, vp, i64, i32, i32, i32, vp, vp, vp]),
        "ivfr_search_static": (ctypes.c_int, [vp, vp, i64, i32, i32, i32, vp, vp, vp]),
        "ivfr_search_trace": (ctypes.c_int, [vp, vp, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "ivfr_search_stats": (ctypes.c_int, [vp] + [ctypes.POINTER(i64)] * 9),
        "ivfr_set_list_sharing": (ctypes.c_int, [vp, i32]),
        "ivfr_set_tuning": (ctypes.c_int, [vp, i32, i32, i32, i32, i32]),
        "ivfr_set_table_mode": (ctypes.c_int, [vp, i32]),
        "ivfr_set_profiling": (ctypes.c_int, [vp, i32]),
        "ivfr_memory_required": (ctypes.c_int, [ctypes.POINTER(Params), i64, i64, i32, i32, i64,
                                                ctypes.POINTER(i64), ctypes.POINTER(i64)]),
        "ivfr_set_memory_limit": (ctypes.c_int, [vp, i64]),
        "ivfr_workspace_info": (ctypes.c_int, [vp] + [ctypes.POINTER(i64)] * 4),
        "ivfr_stage_times": (ctypes.c_int, [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]),
        "ivfr_last_error": (ctypes.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()
EXPORTED = ["ivfr_create", "ivfr_destroy", "ivfr_train", "ivfr_set_codebooks", "ivfr_get_codebooks", "ivfr_add",
            "ivfr_finalize", "ivfr_ntotal", "ivfr_export", "ivfr_import", "ivfr_search", "ivfr_search_static", "ivfr_search_trace",
            "ivfr_search_stats", "ivfr_set_list_sharing", "ivfr_set_tuning", "ivfr_set_profiling", "ivfr_stage_times", "ivfr_last_error",
            "ivfr_memory_required", "ivfr_set_memory_limit", "ivfr_workspace_info", "ivfr_set_table_mode"]


def _check(rc):
    if rc != OK:
        raise IvfrError(rc, lib.ivfr_last_error().decode("utf-8", "replace"))


def _host(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _ptr(x):
    """Address of a host numpy array or a torch tensor (host or device), or None."""
    if x is None:
        return None
    if isinstance(x, np.ndarray):
        assert x.flags["C_CONTIGUOUS"]
        return ctypes.c_void_p(x.ctypes.data)
    assert x.is_contiguous()
    return ctypes.c_void_p(x.data_ptr())


def memory_required(d, c, m, m_refine, N, nq=0, w=1, kprime=1, available=0):
    """(index_bytes, search_bytes) by ivfr_memory_required; raises IvfrError(ERR_OOM) beyond `available`."""
    p = Params(d, c, m, m_refine, 0)
    ib, sb = ctypes.c_int64(), ctypes.c_int64()
    _check(lib.ivfr_memory_required(ctypes.byref(p), N, nq, w, kprime, available, ctypes.byref(ib), ctypes.byref(sb)))
    return ib.value, sb.value


class Index:
    """IVFADC+R index on one GPU (names follow include/ivfadcr.h)."""

    def __init__(self, d, c, m, m_refine, device=0):
        self.d, self.c, self.m, self.m_refine, self.device = d, c, m, m_refine, device
        self._h = ctypes.c_void_p()
        p = Params(d, c, m, m_refine, device)
        _check(lib.ivfr_create(ctypes.byref(p), ctypes.byref(self._h)))

    def close(self):
        if self._h:
            lib.ivfr_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- offline stage
    def train(self, train_u8, iters=10, seed=0):
        """train_u8: uint8 [n, d], numpy (host) or torch (host/device)."""
        n = train_u8.shape[0]
        assert train_u8.shape[1] == self.d and str(train_u8.dtype).endswith("uint8")
        _check(lib.ivfr_train(self._h, _ptr(train_u8), n, iters, seed))

    def set_codebooks(self, coarse, pq, rq=None):
        coarse, pc = _host(coarse, np.float32)
        pq, pp = _host(pq, np.float32)
        assert coarse.shape == (self.c, self.d) and pq.shape == (self.m, 256, self.d // self.m)
        pr = None
        if self.m_refine:
            rq, pr = _host(rq, np.float32)
            assert rq.shape == (self.m_refine, 256, self.d // self.m_refine)
        _check(lib.ivfr_set_codebooks(self._h, pc, pp, pr))

    def get_codebooks(self):
        coarse = np.empty((self.c, self.d), dtype=np.float32)
        pq = np.empty((self.m, 256, self.d // self.m), dtype=np.float32)
        rq = np.empty((self.m_refine, 256, self.d // self.m_refine), dtype=np.float32) if self.m_refine else None
        _check(lib.ivfr_get_codebooks(self._h, _ptr(coarse), _ptr(pq), _ptr(rq)))
        return coarse, pq, rq

    def add(self, x_u8, id_base):
        n = x_u8.shape[0]
        assert n == 0 or (x_u8.shape[1] == self.d and str(x_u8.dtype).endswith("uint8"))
        _check(lib.ivfr_add(self._h, _ptr(x_u8) if n else None, n, id_base))

    def finalize(self):
        _check(lib.ivfr_finalize(self._h))

    @property
    def ntotal(self):
        n = lib.ivfr_ntotal(self._h)
        if n < 0:
            _check(int(n))
        return int(n)

    def export(self):
        N = self.ntotal
        offsets = np.empty(self.c + 1, dtype=np.int64)
        ids = np.empty(N, dtype=np.int32)
        codes = np.empty((N, self.m), dtype=np.uint8)
        rcodes = np.empty((N, self.m_refine), dtype=np.uint8)
        _check(lib.ivfr_export(self._h, _ptr(offsets), _ptr(ids), _ptr(codes),
                               _ptr(rcodes) if self.m_refine else None))
        return offsets, ids, codes, rcodes

    def import_(self, list_offsets, ids, codes, rcodes=None):
        offsets, po = _host(list_offsets, np.int64)
        ids, pi = _host(ids, np.int32)
        codes, pc = _host(codes, np.uint8)
        pr = None
        if self.m_refine:
            rcodes, pr = _host(rcodes, np.uint8)
        _check(lib.ivfr_import(self._h, len(ids), po, pi, pc, pr))

    # ---- query stage
    def search(self, queries, w, kprime, k, stream=None, trace=False):
        """queries: torch fp32 [nq, d] on this index's device.  Returns (ids, dist) torch tensors,
        plus a dict of intermediate results when trace=True."""
        import torch
        assert queries.dtype == torch.float32 and queries.is_cuda and queries.is_contiguous()
        nq = queries.shape[0]
        assert nq == 0 or queries.shape[1] == self.d
        dev = queries.device
        ids = torch.empty((nq, k), dtype=torch.int32, device=dev)
        dist = torch.empty((nq, k), dtype=torch.float32, device=dev)
        st = ctypes.c_void_p(stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream)
        if not trace:
            _check(lib.ivfr_search(self._h, _ptr(queries), nq, w, kprime, k, _ptr(ids), _ptr(dist), st))
            return ids, dist
        t = dict(probe=torch.empty((nq, w), dtype=torch.int32, device=dev),
                 probe_dist=torch.empty((nq, w), dtype=torch.float32, device=dev),
                 short_ids=torch.empty((nq, kprime), dtype=torch.int32, device=dev),
                 short_est=torch.empty((nq, kprime), dtype=torch.float32, device=dev),
                 short_ref=torch.empty((nq, kprime), dtype=torch.float32, device=dev),
                 short_count=torch.empty((nq,), dtype=torch.int32, device=dev))
        _check(lib.ivfr_search_trace(self._h, _ptr(queries), nq, w, kprime, k, _ptr(ids), _ptr(dist),
                                     _ptr(t["probe"]), _ptr(t["probe_dist"]), _ptr(t["short_ids"]),
                                     _ptr(t["short_est"]), _ptr(t["short_ref"]), _ptr(t["short_count"]), st))
        return ids, dist, t

    def search_static(self, queries, w, kprime, k, ids, dist, stream=None):
        """ivfr_search_static: the caller passes the output tensors (int32 [nq, k], fp32 [nq, k]); nothing is
        allocated on the device by this method or by the library."""
        import torch
        assert queries.dtype == torch.float32 and queries.is_cuda and queries.is_contiguous()
        nq = queries.shape[0]
        assert ids.dtype == torch.int32 and dist.dtype == torch.float32 and ids.shape == (nq, k) and dist.shape == (nq, k)
        assert ids.is_contiguous() and dist.is_contiguous()
        st = ctypes.c_void_p(stream if stream is not None else torch.cuda.current_stream(queries.device).cuda_stream)
        _check(lib.ivfr_search_static(self._h, _ptr(queries), nq, w, kprime, k, _ptr(ids), _ptr(dist), st))

    def search_stats(self):
        v = [ctypes.c_int64() for _ in range(9)]
        _check(lib.ivfr_search_stats(self._h, *[ctypes.byref(x) for x in v]))
        names = ("codes_scanned", "pairs", "dense_fallbacks", "codes_streamed", "codes_scanned_shared",
                 "codes_scanned_shared2", "codes_scanned_shared8", "bound_retries", "codes_scanned_shared64")
        return dict(zip(names, [x.value for x in v]))

    def set_list_sharing(self, mode=-1):
        """-1 = 2 for large batches, 0 for small ones (default); 0 = per pair; 1 = fp32 units of four / two;
        2 = also fp16 units of eight; 3 = also matrix-core units of 64."""
        _check(lib.ivfr_set_list_sharing(self._h, int(mode)))

    def set_table_mode(self, mode):
        """0 = one look-up table per (query, list) pair in the workspace; 1 = split tables (per-list and per-query
        terms summed in the scan's prologue)."""
        _check(lib.ivfr_set_table_mode(self._h, int(mode)))

    def set_tuning(self, full_mult=0, cap_mult=0, min_cap=0, batch=0, scan_groups=0):
        _check(lib.ivfr_set_tuning(self._h, full_mult, cap_mult, min_cap, batch, scan_groups))

    def set_memory_limit(self, nbytes):
        """Cap on the device bytes this index may hold in total (0 = none)."""
        _check(lib.ivfr_set_memory_limit(self._h, int(nbytes)))

    def workspace_info(self):
        v = [ctypes.c_int64() for _ in range(4)]
        _check(lib.ivfr_workspace_info(self._h, *[ctypes.byref(x) for x in v]))
        return dict(zip(("index_bytes", "workspace_bytes", "pool_bytes", "batch_reruns"), [x.value for x in v]))

    def set_profiling(self, level=2):
        """0 / False = off, 1 = time the list-scan launches only, 2 / True = time every stage."""
        level = 2 if level is True else (0 if level is False else int(level))
        _check(lib.ivfr_set_profiling(self._h, level))

    STAGES = ("coarse", "probe", "lut", "sample", "scan", "shortlist", "rerank", "final", "scan_shared", "scan_shared2", "scan_shared8", "scan_shared64", "host_enqueue", "host_wait")

    def stage_times(self):
        """Per-stage milliseconds of the last search (after set_profiling) and scan launch count."""
        ms = (ctypes.c_double * len(self.STAGES))()
        n = ctypes.c_int32()
        _check(lib.ivfr_stage_times(self._h, ms, ctypes.byref(n)))
        out = dict(zip(self.STAGES, [float(v) for v in ms]))
        out["scan_launches"] = n.value
        return out
