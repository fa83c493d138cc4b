"""ctypes front end of the CPU oracle (rairs_oracle.c) -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.  It builds the C
file with gcc on first use and never touches the HIP library or the package's binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rairs_oracle.c")
_LIB = os.path.join(_HERE, "librairs_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
                               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Index(C.Structure):
    _fields_ = [
        ("d", C.c_int32), ("M", C.c_int32), ("nlist", C.c_int32), ("raw_is_u8", C.c_int32),
        ("metric", C.c_int32), ("blk", C.c_int32),
        ("ntotal", C.c_int64), ("nblocks", C.c_int64), ("nrefs", C.c_int64),
        ("centroids", C.c_void_p), ("codebook", C.c_void_p), ("codes", C.c_void_p),
        ("ids", C.c_void_p), ("other", C.c_void_p),
        ("list_shared_begin", C.c_void_p), ("list_shared_cnt", C.c_void_p),
        ("list_misc_begin", C.c_void_p), ("list_misc_cnt", C.c_void_p),
        ("list_ref_begin", C.c_void_p), ("list_ref_cnt", C.c_void_p),
        ("ref_owner", C.c_void_p), ("ref_block_begin", C.c_void_p), ("ref_nblocks", C.c_void_p),
        ("raw", C.c_void_p), ("assign", C.c_void_p), ("vec_codes", C.c_void_p),
    ]


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_l2sqr.restype = C.c_float
        _lib.oracle_l2sqr_u8.restype = C.c_float
        _lib.oracle_ip.restype = C.c_float
        _lib.oracle_ip_u8.restype = C.c_float
        _lib.oracle_search.restype = C.c_int
    return _lib


_FIELDS = [("centroids", np.float32), ("codebook", np.float32), ("codes", np.uint8),
           ("ids", np.int64), ("other", np.int32), ("list_shared_begin", np.int64),
           ("list_shared_cnt", np.int32), ("list_misc_begin", np.int64),
           ("list_misc_cnt", np.int32), ("list_ref_begin", np.int64), ("list_ref_cnt", np.int32),
           ("ref_owner", np.int32), ("ref_block_begin", np.int64), ("ref_nblocks", np.int32),
           ("assign", np.int32), ("vec_codes", np.uint8)]


class OracleIndex:
    """Pins the arrays of a host index (any object with the canonical attribute names)."""

    def __init__(self, hx):
        self.keep = {}
        s = _Index()
        s.d, s.M, s.nlist = hx.d, hx.M, hx.nlist
        # metric: "l2" (squared Euclidean distance) or "ip" (inner product); blk: items per block
        self.metric = getattr(hx, "metric", "l2")
        s.metric = {"l2": 0, "ip": 1}[self.metric]
        s.blk = int(hx.ids.shape[1])
        s.ntotal, s.nblocks, s.nrefs = hx.ntotal, hx.ids.shape[0], hx.ref_owner.shape[0]
        for name, dt in _FIELDS:
            a = np.ascontiguousarray(getattr(hx, name), dtype=dt)
            self.keep[name] = a
            setattr(s, name, a.ctypes.data)
        raw = np.ascontiguousarray(hx.raw)
        assert raw.dtype in (np.float32, np.uint8)
        s.raw_is_u8 = int(raw.dtype == np.uint8)
        self.keep["raw"] = raw
        s.raw = raw.ctypes.data
        self.s = s
        self.d, self.M, self.nlist, self.ntotal = hx.d, hx.M, hx.nlist, hx.ntotal
        self.nblocks = int(s.nblocks)


@dataclass
class OracleResult:
    ids: np.ndarray         # [nq][k] i64
    dists: np.ndarray       # [nq][k] f32: squared L2 ascending, or inner products descending
    cand_ids: np.ndarray    # [nq][refine_k] i64 in (score, id) order, -1 padded
    cand_acc: np.ndarray    # [nq][refine_k] i32 16-bit scores, -1 padded
    dco: np.ndarray         # [nq] i64 items scored
    probes: np.ndarray      # [nq][nprobe] i32 in (distance, id) order
    lut: np.ndarray         # [nq][M][16] u8
    push_count: np.ndarray | None = None
    block_count: np.ndarray | None = None


def l2sqr(a: np.ndarray, b: np.ndarray) -> float:
    lib = _load()
    a = np.ascontiguousarray(a, dtype=np.float32)
    if b.dtype == np.uint8:
        b = np.ascontiguousarray(b)
        return float(lib.oracle_l2sqr_u8(C.c_void_p(a.ctypes.data), C.c_void_p(b.ctypes.data),
                                         C.c_int(a.size)))
    b = np.ascontiguousarray(b, dtype=np.float32)
    return float(lib.oracle_l2sqr(C.c_void_p(a.ctypes.data), C.c_void_p(b.ctypes.data),
                                  C.c_int(a.size)))


def ip(a: np.ndarray, b: np.ndarray) -> float:
    """Inner product in the oracle's summation order (b float32 or uint8)."""
    lib = _load()
    a = np.ascontiguousarray(a, dtype=np.float32)
    if b.dtype == np.uint8:
        b = np.ascontiguousarray(b)
        return float(lib.oracle_ip_u8(C.c_void_p(a.ctypes.data), C.c_void_p(b.ctypes.data), C.c_int(a.size)))
    b = np.ascontiguousarray(b, dtype=np.float32)
    return float(lib.oracle_ip(C.c_void_p(a.ctypes.data), C.c_void_p(b.ctypes.data), C.c_int(a.size)))


def coarse(ox: OracleIndex, q: np.ndarray, nprobe: int):
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float32)
    lists = np.empty(nprobe, dtype=np.int32)
    dists = np.empty(nprobe, dtype=np.float32)
    lib.oracle_coarse(C.byref(ox.s), C.c_void_p(q.ctypes.data), C.c_int(nprobe),
                      C.c_void_p(lists.ctypes.data), C.c_void_p(dists.ctypes.data))
    return lists, dists


def lut(ox: OracleIndex, q: np.ndarray):
    """Float table T[M][16], its 8-bit quantisation, sum of per-subspace minima, scale."""
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float32)
    T = np.empty((ox.M, 16), dtype=np.float32)
    u8 = np.empty((ox.M, 16), dtype=np.uint8)
    bias = C.c_float()
    scale = C.c_float()
    lib.oracle_lut(C.byref(ox.s), C.c_void_p(q.ctypes.data), C.c_void_p(T.ctypes.data),
                   C.c_void_p(u8.ctypes.data), C.byref(bias), C.byref(scale))
    return T, u8, bias.value, scale.value


def pq_encode(codebook: np.ndarray, x: np.ndarray) -> np.ndarray:
    """PQEncoding (Alg. 1): packed codes [n][M/2] of the rows of x for codebook [M][16][d/M]."""
    lib = _load()
    cb = np.ascontiguousarray(codebook, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.float32)
    M, ksub, dsub = cb.shape
    assert ksub == 16 and x.shape[1] == M * dsub and M % 2 == 0
    out = np.empty((x.shape[0], M // 2), dtype=np.uint8)
    lib.oracle_pq_encode(C.c_void_p(cb.ctypes.data), C.c_int(M * dsub), C.c_int(M),
                         C.c_void_p(x.ctypes.data), C.c_int64(x.shape[0]), C.c_void_p(out.ctypes.data))
    return out


def rair_assign(centroids: np.ndarray, x: np.ndarray, n_cands: int = 10, lam: float = 0.5,
                strict: bool = True) -> np.ndarray:
    """RairAssign (Alg. 3): [n][2] list ids per vector, the smaller id first."""
    lib = _load()
    c = np.ascontiguousarray(centroids, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert c.shape[1] == x.shape[1] and n_cands >= 1
    out = np.empty((x.shape[0], 2), dtype=np.int32)
    lib.oracle_rair_assign(C.c_void_p(c.ctypes.data), C.c_int(c.shape[0]), C.c_int(c.shape[1]),
                           C.c_void_p(x.ctypes.data), C.c_int64(x.shape[0]), C.c_int(n_cands),
                           C.c_double(lam), C.c_int(int(strict)), C.c_void_p(out.ctypes.data))
    return out


def search(ox: OracleIndex, queries: np.ndarray, k: int, nprobe: int, refine_k: int,
           layout: str = "seil", nthreads: int = 0, trace: bool = False) -> OracleResult:
    """layout "seil": Alg. 5 on the SEIL directory; "naive": union of probed lists' members."""
    lib = _load()
    queries = np.ascontiguousarray(queries, dtype=np.float32)
    nq = queries.shape[0]
    assert queries.shape[1] == ox.d
    r = OracleResult(
        ids=np.empty((nq, k), dtype=np.int64), dists=np.empty((nq, k), dtype=np.float32),
        cand_ids=np.empty((nq, refine_k), dtype=np.int64),
        cand_acc=np.empty((nq, refine_k), dtype=np.int32), dco=np.empty(nq, dtype=np.int64),
        probes=np.empty((nq, nprobe), dtype=np.int32),
        lut=np.empty((nq, ox.M, 16), dtype=np.uint8))
    pc = bc = None
    if trace:
        r.push_count = np.zeros((nq, ox.ntotal), dtype=np.int32)
        r.block_count = np.zeros((nq, ox.nblocks), dtype=np.int32)
        pc, bc = r.push_count.ctypes.data, r.block_count.ctypes.data
    rc = lib.oracle_search(
        C.byref(ox.s), C.c_void_p(queries.ctypes.data), C.c_int64(nq), C.c_int(k),
        C.c_int(nprobe), C.c_int(refine_k), C.c_int(0 if layout == "seil" else 1),
        C.c_int(nthreads), C.c_void_p(r.ids.ctypes.data), C.c_void_p(r.dists.ctypes.data),
        C.c_void_p(r.cand_ids.ctypes.data), C.c_void_p(r.cand_acc.ctypes.data),
        C.c_void_p(r.dco.ctypes.data), C.c_void_p(r.probes.ctypes.data),
        C.c_void_p(r.lut.ctypes.data), C.c_void_p(pc), C.c_void_p(bc))
    if rc != 0:
        raise ValueError("oracle_search: invalid arguments")
    return r


def num_threads() -> int:
    return int(_load().oracle_num_threads())
