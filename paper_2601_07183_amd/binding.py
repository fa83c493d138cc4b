"""Thin Python binding of librairs.so: argument marshalling only.

Function names mirror include/rairs.h.  PyTorch supplies device memory and the stream; every
step of the search runs in the library's HIP kernels.  There is no CPU fallback: if the shared
library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librairs.so")
_lib = None

STAGES = ("coarse", "lut", "scan", "refine", "scan_kernel")
MAX_REFINE_K = 1024
MAX_NPROBE = 4096

EXPORTS = ("rairs_index_upload", "rairs_search", "rairs_free", "rairs_workspace_bytes", "rairs_set_workspace",
           "rairs_search_noalloc", "rairs_graph_create", "rairs_graph_launch", "rairs_graph_free",
           "rairs_coarse", "rairs_lut",
           "rairs_scan", "rairs_refine", "rairs_set_scan_mode", "rairs_set_profiling", "rairs_get_stage_ms",
           "rairs_get_stage_ms_mean",
           "rairs_get_dco", "rairs_get_scan_stats", "rairs_scan_kernel_name", "rairs_index_bytes", "rairs_pq_encode", "rairs_assign",
           "rairs_last_error")


PROFILE_STAGES, PROFILE_SCAN_KERNEL = 1, 2


class RairsError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"rairs error {code}: {msg}")
        self.code = code


class _HostIndex(C.Structure):
    _fields_ = [
        ("d", C.c_int32), ("M", C.c_int32), ("nbits", C.c_int32), ("nlist", C.c_int32),
        ("blk", C.c_int32), ("raw_is_u8", C.c_int32),
        ("ntotal", C.c_int64), ("nblocks", C.c_int64), ("nrefs", C.c_int64),
        ("centroids", C.c_void_p), ("codebook", C.c_void_p), ("codes", C.c_void_p),
        ("ids", C.c_void_p), ("other", C.c_void_p),
        ("list_shared_begin", C.c_void_p), ("list_shared_cnt", C.c_void_p),
        ("list_misc_begin", C.c_void_p), ("list_misc_cnt", C.c_void_p),
        ("list_ref_begin", C.c_void_p), ("list_ref_cnt", C.c_void_p),
        ("ref_owner", C.c_void_p), ("ref_block_begin", C.c_void_p), ("ref_nblocks", C.c_void_p),
        ("raw", C.c_void_p), ("metric", C.c_int32),
    ]


def load() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with "
                "`python -m paper_2601_07183_amd.build_ext` (there is no fallback path)")
        lib = C.CDLL(LIB_PATH)
        lib.rairs_last_error.restype = C.c_char_p
        lib.rairs_workspace_bytes.restype = C.c_size_t
        lib.rairs_scan_kernel_name.restype = C.c_char_p
        for name in EXPORTS:
            getattr(lib, name)
        _lib = lib
    return _lib


def _check(rc: int):
    if rc != 0:
        raise RairsError(rc, load().rairs_last_error().decode())


def _stream_ptr(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str) -> C.c_void_p:
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{name}: expected a contiguous device tensor of {dtype}")
    return C.c_void_p(t.data_ptr())


_ARRAYS = [("centroids", np.float32), ("codebook", np.float32), ("codes", np.uint8),
           ("ids", np.int64), ("other", np.int32), ("list_shared_begin", np.int64),
           ("list_shared_cnt", np.int32), ("list_misc_begin", np.int64),
           ("list_misc_cnt", np.int32), ("list_ref_begin", np.int64), ("list_ref_cnt", np.int32),
           ("ref_owner", np.int32), ("ref_block_begin", np.int64), ("ref_nblocks", np.int32)]


def pq_encode(codebook: torch.Tensor, vectors: torch.Tensor, stream=None) -> torch.Tensor:
    """rairs_pq_encode: packed codes [n][M/2] of device vectors [n][d] for a device codebook [M][16][d/M]."""
    lib = load()
    M, ksub, dsub = codebook.shape
    if ksub != 16 or vectors.ndim != 2 or vectors.shape[1] != M * dsub:
        raise ValueError("codebook must be [M][16][d/M] and vectors [n][d]")
    n = vectors.shape[0]
    codes = torch.empty((n, M // 2), dtype=torch.uint8, device=vectors.device)
    _check(lib.rairs_pq_encode(_dev(codebook, torch.float32, "codebook"), C.c_int(M * dsub), C.c_int(M),
                               _dev(vectors, torch.float32, "vectors") if n else C.c_void_p(0),
                               C.c_int64(n), _dev(codes, torch.uint8, "codes") if n else C.c_void_p(0),
                               _stream_ptr(stream)))
    return codes


def host_struct(hx):
    """ctypes view of a host index object (attributes named as in rairs_host_index_t)."""
    keep = []
    s = _HostIndex()
    s.d, s.M, s.nbits, s.nlist, s.blk = hx.d, hx.M, 4, hx.nlist, int(np.shape(hx.ids)[1])
    s.metric = {"l2": 0, "ip": 1}[getattr(hx, "metric", "l2")]
    s.ntotal, s.nblocks, s.nrefs = hx.ntotal, hx.ids.shape[0], hx.ref_owner.shape[0]
    for name, dt in _ARRAYS:
        a = np.ascontiguousarray(getattr(hx, name), dtype=dt)
        keep.append(a)
        setattr(s, name, a.ctypes.data)
    raw = np.ascontiguousarray(hx.raw)
    if raw.dtype not in (np.float32, np.uint8):
        raise TypeError("raw vectors must be float32 or uint8")
    s.raw_is_u8 = int(raw.dtype == np.uint8)
    s.raw = raw.ctypes.data
    keep.append(raw)
    return s, keep


class SearchGraph:
    """A captured search (rairs_graph_create ... rairs_graph_free); keeps its tensors alive."""

    def __init__(self, lib, g, tensors):
        self._lib, self._g, self._tensors = lib, g, tensors

    def launch(self, stream=None):
        _check(self._lib.rairs_graph_launch(self._g, _stream_ptr(stream)))

    def free(self):
        if self._g:
            _check(self._lib.rairs_graph_free(self._g))
            self._g = C.c_void_p()

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class Index:
    """Device-resident RAIRS index (rairs_index_upload ... rairs_free)."""

    def __init__(self, hx, stream=None):
        self._h = C.c_void_p()
        self._lib = load()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the search path has no CPU implementation")
        s, keep = host_struct(hx)
        _check(self._lib.rairs_index_upload(C.byref(s), _stream_ptr(stream), C.byref(self._h)))
        del keep
        self.d, self.M, self.nlist, self.ntotal = hx.d, hx.M, hx.nlist, hx.ntotal
        self._ws = None                 # torch tensor that serves as the handle's workspace

    # --- workspace: device memory comes from PyTorch ------------------------------------------
    def workspace_bytes(self, nq: int, nprobe: int, refine_k: int) -> int:
        """rairs_workspace_bytes (0 for an empty batch; raises on arguments the search rejects)."""
        n = int(self._lib.rairs_workspace_bytes(self._h, C.c_int64(nq), C.c_int(nprobe), C.c_int(refine_k)))
        if n == 0 and nq > 0:
            raise RairsError(-1, self._lib.rairs_last_error().decode())
        return n

    def set_workspace(self, ws):
        """rairs_set_workspace: a uint8 device tensor (kept alive here), or None for the handle's own."""
        if ws is None:
            _check(self._lib.rairs_set_workspace(self._h, C.c_void_p(0), C.c_size_t(0)))
        else:
            _check(self._lib.rairs_set_workspace(self._h, _dev(ws, torch.uint8, "workspace"),
                                                 C.c_size_t(ws.numel())))
        self._ws = ws

    def _reserve(self, nq: int, nprobe: int, refine_k: int):
        """Give the handle a torch-allocated workspace large enough for this call (arguments that
        the library rejects are left to the call itself, which reports them)."""
        if nq <= 0 or self._ws is False:
            return
        need = int(self._lib.rairs_workspace_bytes(self._h, C.c_int64(nq), C.c_int(nprobe), C.c_int(refine_k)))
        if need and (self._ws is None or self._ws.numel() < need):
            torch.cuda.current_stream().synchronize()     # nothing of this handle is in flight
            self._ws = None
            self.set_workspace(torch.empty(need, dtype=torch.uint8, device="cuda"))

    def use_own_workspace(self):
        """Let the library allocate and grow its workspace itself (hipMalloc inside the handle)."""
        self.set_workspace(None)
        self._ws = False

    def free(self):
        if self._h:
            _check(self._lib.rairs_free(self._h))
            self._h = C.c_void_p()
            self._ws = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    # --- rairs_search ---------------------------------------------------------------------
    def search(self, queries: torch.Tensor, k: int, nprobe: int, refine_k: int, out_ids=None,
               out_dists=None, stream=None):
        nq = queries.shape[0]
        if out_ids is None:
            out_ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
        if out_dists is None:
            out_dists = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
        self._reserve(nq, nprobe, refine_k)
        _check(self._lib.rairs_search(
            self._h, _dev(queries, torch.float32, "queries"), C.c_int64(nq), C.c_int(k),
            C.c_int(nprobe), C.c_int(refine_k), _dev(out_ids, torch.int64, "out_ids"),
            _dev(out_dists, torch.float32, "out_dists"), _stream_ptr(stream)))
        return out_ids, out_dists

    def search_noalloc(self, queries: torch.Tensor, k: int, nprobe: int, refine_k: int, out_ids,
                       out_dists, stream=None):
        """rairs_search_noalloc: the caller supplies the outputs; scratch memory is the library's
        static device array."""
        _check(self._lib.rairs_search_noalloc(
            self._h, _dev(queries, torch.float32, "queries"), C.c_int64(queries.shape[0]), C.c_int(k),
            C.c_int(nprobe), C.c_int(refine_k), _dev(out_ids, torch.int64, "out_ids"),
            _dev(out_dists, torch.float32, "out_dists"), _stream_ptr(stream)))
        return out_ids, out_dists

    def graph(self, queries: torch.Tensor, k: int, nprobe: int, refine_k: int, out_ids, out_dists, stream):
        """rairs_graph_create: returns a SearchGraph that replays this search on the given tensors."""
        g = C.c_void_p()
        _check(self._lib.rairs_graph_create(
            self._h, _dev(queries, torch.float32, "queries"), C.c_int64(queries.shape[0]), C.c_int(k),
            C.c_int(nprobe), C.c_int(refine_k), _dev(out_ids, torch.int64, "out_ids"),
            _dev(out_dists, torch.float32, "out_dists"), _stream_ptr(stream), C.byref(g)))
        return SearchGraph(self._lib, g, (queries, out_ids, out_dists))

    # --- stages ---------------------------------------------------------------------------
    def coarse(self, queries: torch.Tensor, nprobe: int, stream=None):
        nq = queries.shape[0]
        self._reserve(nq, nprobe, 1)
        ids = torch.empty((nq, nprobe), dtype=torch.int32, device=queries.device)
        dists = torch.empty((nq, nprobe), dtype=torch.float32, device=queries.device)
        _check(self._lib.rairs_coarse(self._h, _dev(queries, torch.float32, "queries"),
                                      C.c_int64(nq), C.c_int(nprobe), _dev(ids, torch.int32, "ids"),
                                      _dev(dists, torch.float32, "dists"), _stream_ptr(stream)))
        return ids, dists

    def lut(self, queries: torch.Tensor, stream=None):
        nq = queries.shape[0]
        lut = torch.empty((nq, self.M, 16), dtype=torch.uint8, device=queries.device)
        bias = torch.empty((nq,), dtype=torch.float32, device=queries.device)
        scale = torch.empty((nq,), dtype=torch.float32, device=queries.device)
        _check(self._lib.rairs_lut(self._h, _dev(queries, torch.float32, "queries"), C.c_int64(nq),
                                   _dev(lut, torch.uint8, "lut"), _dev(bias, torch.float32, "bias"),
                                   _dev(scale, torch.float32, "scale"), _stream_ptr(stream)))
        return lut, bias, scale

    def scan(self, lut: torch.Tensor, probe_ids: torch.Tensor, refine_k: int, stream=None):
        nq, nprobe = probe_ids.shape
        self._reserve(nq, nprobe, refine_k)
        cand = torch.empty((nq, refine_k), dtype=torch.int64, device=lut.device)
        score = torch.empty((nq, refine_k), dtype=torch.int32, device=lut.device)
        dco = torch.empty((nq,), dtype=torch.int64, device=lut.device)
        _check(self._lib.rairs_scan(self._h, _dev(lut, torch.uint8, "lut"),
                                    _dev(probe_ids, torch.int32, "probe_ids"), C.c_int64(nq),
                                    C.c_int(nprobe), C.c_int(refine_k),
                                    _dev(cand, torch.int64, "cand"), _dev(score, torch.int32, "score"),
                                    _dev(dco, torch.int64, "dco"), _stream_ptr(stream)))
        return cand, score, dco

    def refine(self, queries: torch.Tensor, cand_ids: torch.Tensor, k: int, stream=None):
        nq, refine_k = cand_ids.shape
        ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
        dists = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
        _check(self._lib.rairs_refine(self._h, _dev(queries, torch.float32, "queries"),
                                      _dev(cand_ids, torch.int64, "cand_ids"), C.c_int64(nq),
                                      C.c_int(refine_k), C.c_int(k), _dev(ids, torch.int64, "ids"),
                                      _dev(dists, torch.float32, "dists"), _stream_ptr(stream)))
        return ids, dists

    def set_scan_mode(self, exact: bool):
        _check(self._lib.rairs_set_scan_mode(self._h, C.c_int(1 if exact else 0)))

    # --- measurement ----------------------------------------------------------------------
    def set_profiling(self, level):
        """False / 0: off; True / PROFILE_STAGES: every stage; PROFILE_SCAN_KERNEL: the scan kernel only."""
        _check(self._lib.rairs_set_profiling(self._h, C.c_int(int(level))))

    def stage_ms(self) -> dict:
        ms = (C.c_float * len(STAGES))()
        _check(self._lib.rairs_get_stage_ms(self._h, ms))
        return dict(zip(STAGES, [float(x) for x in ms]))

    def stage_ms_mean(self, last_n: int) -> dict:
        ms = (C.c_float * len(STAGES))()
        _check(self._lib.rairs_get_stage_ms_mean(self._h, C.c_int(last_n), ms))
        return dict(zip(STAGES, [float(x) for x in ms]))

    def assign(self, vectors: torch.Tensor, n_cands: int = 10, lam: float = 0.5, strict: bool = True,
               stream=None) -> torch.Tensor:
        """rairs_assign: [n][2] list ids (smaller first) of device vectors [n][d]."""
        n = vectors.shape[0]
        self._reserve(n, max(1, min(n_cands, self.nlist)), 1)
        out = torch.empty((n, 2), dtype=torch.int32, device=vectors.device)
        _check(self._lib.rairs_assign(self._h, _dev(vectors, torch.float32, "vectors") if n else C.c_void_p(0),
                                      C.c_int64(n), C.c_int(n_cands), C.c_double(lam), C.c_int(int(strict)),
                                      _dev(out, torch.int32, "pairs") if n else C.c_void_p(0),
                                      _stream_ptr(stream)))
        return out

    def dco(self, nq: int) -> np.ndarray:
        out = np.empty(nq, dtype=np.int64)
        _check(self._lib.rairs_get_dco(self._h, C.c_void_p(out.ctypes.data), C.c_int64(nq)))
        return out

    def scan_stats(self) -> dict:
        st = (C.c_int64 * 5)()
        _check(self._lib.rairs_get_scan_stats(self._h, st))
        return dict(redone=int(st[0]), survivors=int(st[1]), max_survivors=int(st[2]),
                    queries=int(st[3]), logged=int(st[4]))

    def scan_kernel_name(self) -> str:
        return self._lib.rairs_scan_kernel_name(self._h).decode()

    def bytes(self):
        a, b = C.c_int64(), C.c_int64()
        _check(self._lib.rairs_index_bytes(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value
