"""The C-ABI library loads and exports what include/rairs.h declares; host-side argument checks
answer without touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2601_07183_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "rairs.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rairs_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = binding.load()
    names = _declared()
    assert "rairs_index_upload" in names and "rairs_search" in names and "rairs_free" in names
    for n in names:
        assert getattr(lib, n) is not None
    assert set(names) == set(binding.EXPORTS)


def test_null_and_invalid_arguments_are_rejected_on_the_host(small_index):
    lib = binding.load()
    h = C.c_void_p()
    assert lib.rairs_index_upload(None, None, C.byref(h)) == -1
    assert b"NULL" in lib.rairs_last_error()
    assert lib.rairs_search(None, None, C.c_int64(1), 1, 1, 1, None, None, None) == -1
    assert lib.rairs_free(None) == 0
    base, hx = small_index
    s, keep = binding.host_struct(hx)
    for field, bad in (("nbits", 8), ("blk", 64), ("M", 7), ("nlist", 0), ("ntotal", -1)):
        old = getattr(s, field)
        setattr(s, field, bad)
        assert lib.rairs_index_upload(C.byref(s), None, C.byref(h)) == -1, field
        assert not h.value
        setattr(s, field, old)
    # a reference entry that points outside its owner's shared blocks
    if hx.nrefs:
        bad = np.array(keep[12], copy=True)
        bad[0] = 10 ** 9
        old = s.ref_block_begin
        s.ref_block_begin = bad.ctypes.data
        assert lib.rairs_index_upload(C.byref(s), None, C.byref(h)) == -1
        s.ref_block_begin = old
    # a vector id beyond ntotal
    bad_ids = np.array(keep[3], copy=True)
    bad_ids[0, 0] = hx.ntotal
    s.ids = bad_ids.ctypes.data
    assert lib.rairs_index_upload(C.byref(s), None, C.byref(h)) == -1
    assert b"id out of range" in lib.rairs_last_error()


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(FileNotFoundError):
        binding.load()
