"""The entry point that allocates nothing: rairs_search_noalloc runs in a static device array and
must return what rairs_search returns."""
import ctypes as C

import numpy as np
import pytest

from oracle import oracle
from paper_2601_07183_amd import datagen, index_build as ib

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_search_noalloc_matches_search_on_two_calls_in_a_row():
    from paper_2601_07183_amd import binding
    lib = binding.load()
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    w = datagen.WORKLOADS["tiny"]
    base = datagen.make_base(w)
    q = datagen.make_queries(w)
    hx = ib.build_index(base, w.nlist, w.M, seed=w.seed)
    ix = binding.Index(hx)
    try:
        # the second call is smaller (fewer queries, fewer probes, smaller bigK) and runs in the
        # same array, which still holds the first call's contents
        for nq, k, nprobe, refine_k in ((200, 10, 16, 40), (37, 5, 4, 20)):
            print(f"case: noalloc nq={nq} k={k} nprobe={nprobe} refine_k={refine_k}", flush=True)
            dq = torch.from_numpy(q[:nq]).cuda()
            ref_ids, ref_d = ix.search(dq, k, nprobe, refine_k)
            torch.cuda.synchronize()
            ids = torch.full((nq, k), -7, dtype=torch.int64, device="cuda")
            dists = torch.zeros((nq, k), dtype=torch.float32, device="cuda")
            rc = lib.rairs_search_noalloc(
                ix._h, C.c_void_p(dq.data_ptr()), C.c_int64(nq), C.c_int(k), C.c_int(nprobe),
                C.c_int(refine_k), C.c_void_p(ids.data_ptr()), C.c_void_p(dists.data_ptr()),
                C.c_void_p(torch.cuda.current_stream().cuda_stream))
            assert rc == 0, lib.rairs_last_error()
            torch.cuda.synchronize()
            # bit-exact against the existing entry point (ids) and the same distance bits
            assert (ids == ref_ids).all()
            assert (dists == ref_d).all()
            # and against the oracle, to the usual bar
            want = oracle.search(oracle.OracleIndex(hx), q[:nq], k, nprobe, refine_k)
            assert (ids.cpu().numpy() == want.ids).all()
            assert (np.abs(dists.cpu().numpy() - want.dists) <= 1e-5 * np.abs(want.dists)).all()
            assert (ix.dco(nq) == want.dco).all()
        # beyond the array's size: a clear error, nothing enqueued
        big = torch.zeros((40000, hx.d), dtype=torch.float32, device="cuda")
        ids = torch.full((40000, 10), -7, dtype=torch.int64, device="cuda")
        dists = torch.zeros((40000, 10), dtype=torch.float32, device="cuda")
        rc = lib.rairs_search_noalloc(
            ix._h, C.c_void_p(big.data_ptr()), C.c_int64(40000), C.c_int(10), C.c_int(16), C.c_int(40),
            C.c_void_p(ids.data_ptr()), C.c_void_p(dists.data_ptr()),
            C.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == -5 and b"static array" in lib.rairs_last_error()
        torch.cuda.synchronize()
        assert (ids == -7).all()
    finally:
        ix.free()
