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


def _upload_rc(lib, hx, **replaced):
    """Return code and message of rairs_index_upload for hx with some arrays replaced (host side:
    validation comes before the first GPU call)."""
    class View:
        pass
    v = View()
    v.__dict__.update(hx.__dict__)
    v.__dict__.update(replaced)
    s, keep = binding.host_struct(v)
    h = C.c_void_p()
    rc = lib.rairs_index_upload(C.byref(s), None, C.byref(h))
    assert rc != 0 and not h.value
    return rc, lib.rairs_last_error().decode()


def test_layout_rules_are_checked_at_upload(small_index, small_index_nonstrict):
    # Section 5.1's structure, which the scan relies on: leftovers of cell (i, j) sit in both lists
    # as twins with the same code, shared blocks carry no tags, owners have the smaller id, blocks
    # belong to one list.  Each broken rule must come back as RAIRS_EINVAL.
    lib = binding.load()
    for base, hx in (small_index, small_index_nonstrict):
        other = hx.other.reshape(-1)
        ids = hx.ids.reshape(-1)
        misc = np.zeros(hx.nblocks, dtype=bool)
        for L in range(hx.nlist):
            misc[hx.list_misc_begin[L]:hx.list_misc_begin[L] + hx.list_misc_cnt[L]] = True
        own = np.repeat(np.arange(hx.nlist), hx.list_shared_cnt + hx.list_misc_cnt)
        blk_list = np.full(hx.nblocks, -1)
        for L in range(hx.nlist):
            b0 = hx.list_shared_begin[L]
            blk_list[b0:b0 + hx.list_shared_cnt[L] + hx.list_misc_cnt[L]] = L
        slot_list = np.repeat(blk_list, 32)
        twin = np.flatnonzero(np.repeat(misc, 32) & (ids >= 0) & (other != slot_list))
        assert twin.size                                   # the fixture has two-list cells
        t = int(twin[0])
        # a twin whose code differs
        codes = hx.codes.copy()
        codes.reshape(-1, hx.M // 2)[t, 0] ^= 1
        rc, msg = _upload_rc(lib, hx, codes=codes)
        assert rc == -1 and "not twins" in msg
        # a twin that is missing (its slot emptied would break density; retag it as stored once instead)
        o2 = hx.other.copy()
        o2.reshape(-1)[t] = slot_list[t]
        rc, msg = _upload_rc(lib, hx, other=o2)
        assert rc == -1 and ("no twin" in msg or "more than once" in msg or "more often" in msg)
        # a twin tagged with a third list
        o3 = hx.other.copy()
        third = next(L for L in range(hx.nlist) if L not in (slot_list[t], other[t]))
        o3.reshape(-1)[t] = third
        rc, msg = _upload_rc(lib, hx, other=o3)
        assert rc == -1
        # a tag in a shared block
        sh = np.flatnonzero(~np.repeat(misc, 32) & (ids >= 0) & (slot_list >= 0))
        if sh.size:
            o4 = hx.other.copy()
            o4.reshape(-1)[sh[0]] = 0
            rc, msg = _upload_rc(lib, hx, other=o4)
            assert rc == -1 and "shared block" in msg
            # an id stored twice
            i5 = hx.ids.copy()
            i5.reshape(-1)[sh[0]] = ids[t]
            rc, msg = _upload_rc(lib, hx, ids=i5)
            assert rc == -1
        # overlapping list ranges
        big = int(np.argmax(hx.list_shared_cnt + hx.list_misc_cnt))
        nxt = (big + 1) % hx.nlist
        sb = hx.list_shared_begin.copy()
        mb = hx.list_misc_begin.copy()
        sb[nxt] = hx.list_shared_begin[big]
        mb[nxt] = sb[nxt] + hx.list_shared_cnt[nxt]
        if hx.list_shared_cnt[nxt] + hx.list_misc_cnt[nxt] > 0:
            rc, msg = _upload_rc(lib, hx, list_shared_begin=sb, list_misc_begin=mb)
            assert rc == -1
        # a reference entry whose owner is not the smaller list
        if hx.nrefs:
            L = int(np.flatnonzero(hx.list_ref_cnt)[0])
            ro = hx.ref_owner.copy()
            ro[hx.list_ref_begin[L]] = L
            rc, msg = _upload_rc(lib, hx, ref_owner=ro)
            assert rc == -1 and "smaller list id" in msg


def test_workspace_calls_check_their_arguments_on_the_host():
    lib = binding.load()
    assert lib.rairs_workspace_bytes(None, C.c_int64(10), 1, 10) == 0
    assert lib.rairs_set_workspace(None, None, C.c_size_t(0)) == -1
    assert lib.rairs_search_noalloc(None, None, C.c_int64(1), 1, 1, 1, None, None, None) == -1


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(FileNotFoundError):
        binding.load()
