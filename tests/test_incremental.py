"""Later insertion batches and deletion (Section 5.1's rules for a second batch; the deletion rule
of the implementation paragraph of Section 6.1), on the CPU.

The mutated layouts are checked three ways: against the structural rules the paper states, against
the plain definition of the candidate set (members of the probed lists that are still in the
index, each once) through the oracle's two routes, and against exact k nearest neighbours over the
vectors that remain when everything is probed and refined.
"""
import numpy as np
import pytest

from oracle import oracle
from paper_2601_07183_amd import datagen, index_build as ib

BLK = 32


def clumped(seed, n, d, integer=False):
    base = datagen.random_vectors(seed, n, d)
    g = np.random.Generator(np.random.PCG64(seed + 99))
    centers = g.uniform(-1, 1, size=(8, d)).astype(np.float32)
    base = (centers[g.integers(0, 8, size=n)] + 0.25 * base).astype(np.float32)
    if integer:
        base = np.clip(np.rint(base * 60 + 128), 0, 255).astype(np.float32)
    return base


def queries(seed, nq, d, integer=False):
    q = datagen.random_vectors(seed + 1000, nq, d)
    if integer:
        q = np.clip(np.rint(q * 60 + 128), 0, 255).astype(np.float32)
    return q


def check_structure(hx, live, shared_full=True):
    """The rules every layout keeps: where each live vector sits, and which slots may be empty."""
    nlist = hx.nlist
    ids, other = hx.ids, hx.other
    in_own = [dict() for _ in range(nlist)]          # id -> "shared" / "misc" for blocks stored in l
    for l in range(nlist):
        sb, sc = int(hx.list_shared_begin[l]), int(hx.list_shared_cnt[l])
        mb, mc = int(hx.list_misc_begin[l]), int(hx.list_misc_cnt[l])
        assert mb == sb + sc
        for b in range(sb, sb + sc):
            assert (other[b] == -1).all()
            if shared_full:
                assert (ids[b] >= 0).all()
            for x in ids[b][ids[b] >= 0]:
                assert int(x) not in in_own[l]
                in_own[l][int(x)] = "shared"
        flat = ids[mb:mb + mc].reshape(-1)
        nvalid = int((flat >= 0).sum())
        # miscellaneous items are dense: only the tail of the last block is empty, and no block is
        # kept that holds nothing
        assert (flat[:nvalid] >= 0).all() and (flat[nvalid:] < 0).all()
        assert mc == (nvalid + BLK - 1) // BLK
        for b in range(mb, mb + mc):
            for s in range(BLK):
                x = int(ids[b, s])
                if x >= 0:
                    assert x not in in_own[l]
                    in_own[l][x] = "misc"
                    a = hx.assign[x]
                    assert l in a and other[b, s] == (a[0] if a[1] == l else a[1])
    via_ref = [set() for _ in range(nlist)]
    for l in range(nlist):
        rb, rc = int(hx.list_ref_begin[l]), int(hx.list_ref_cnt[l])
        for r in range(rb, rb + rc):
            o, b0, nb = int(hx.ref_owner[r]), int(hx.ref_block_begin[r]), int(hx.ref_nblocks[r])
            assert o < l and nb >= 1
            assert hx.list_shared_begin[o] <= b0 and b0 + nb <= hx.list_shared_begin[o] + hx.list_shared_cnt[o]
            for x in ids[b0:b0 + nb].reshape(-1):
                if x >= 0:
                    assert tuple(hx.assign[x]) == (o, l)     # the blocks hold cell (o, l) only
                    assert int(x) not in via_ref[l]
                    via_ref[l].add(int(x))
    seen = set()
    for l in range(nlist):
        seen |= set(in_own[l]) | via_ref[l]
    assert seen == set(np.flatnonzero(live).tolist())
    for x in np.flatnonzero(live):
        a0, a1 = (int(t) for t in hx.assign[x])
        assert a0 <= a1
        x = int(x)
        if a0 == a1:
            assert x in in_own[a0] and x not in via_ref[a0]
        elif in_own[a0].get(x) == "shared":                  # stored once, reached from a1 by reference
            assert x in via_ref[a1] and x not in in_own[a1]
        else:
            assert in_own[a0].get(x) == "misc" and in_own[a1].get(x) == "misc"
    for x in np.flatnonzero(~live):
        assert tuple(hx.assign[x]) == (-1, -1)


def check_search(hx, base, live, integer, seed):
    ox = oracle.OracleIndex(hx)
    q = queries(seed, 30, hx.d, integer)
    for nprobe in (1, 3, 8, hx.nlist):
        a = oracle.search(ox, q, 10, nprobe, 60, layout="seil")
        b = oracle.search(ox, q, 10, nprobe, 60, layout="naive")
        assert (a.cand_ids == b.cand_ids).all() and (a.cand_acc == b.cand_acc).all()
        assert (a.ids == b.ids).all() and (a.dists == b.dists).all()
        got = a.cand_ids[a.cand_ids >= 0]
        assert live[got].all()
    if integer:
        # everything probed and refined: exact kNN over what is left (integer data: exact ties too)
        r = oracle.search(ox, q, 10, hx.nlist, hx.ntotal)
        keep = np.flatnonzero(live)
        d2 = ((q[:, None, :].astype(np.float64) - base[keep][None, :, :].astype(np.float64)) ** 2).sum(-1)
        for i in range(len(q)):
            order = keep[np.lexsort((keep, d2[i]))][:10]
            assert (r.ids[i] == order).all()


def three_batches(seed, integer, strict):
    base = clumped(seed, 3000, 16, integer)
    hx = ib.build_index(base[:1800], 16, 8, seed=seed, coarse_iters=8, pq_iters=8, strict=strict)
    steps = [hx]
    for lo, hi in ((1800, 2500), (2500, 3000)):
        hx = ib.append_batch(hx, base[lo:hi], strict=strict)
        steps.append(hx)
    return base, steps


@pytest.mark.parametrize("strict", [True, False])
def test_append_keeps_the_rules_and_the_candidate_set(strict):
    base, steps = three_batches(21, True, strict)
    for hx in steps:
        live = np.ones(hx.ntotal, dtype=bool)
        check_structure(hx, live)
        check_search(hx, base[:hx.ntotal], live, True, 3)


def test_append_adds_entries_after_the_old_ones_and_fills_the_last_block_first():
    base, (h0, h1, h2) = three_batches(22, False, True)
    for old, new in ((h0, h1), (h1, h2)):
        grew = 0
        for l in range(old.nlist):
            # shared blocks and reference entries of the earlier batches come first, unchanged
            sc = int(old.list_shared_cnt[l])
            a = old.ids[old.list_shared_begin[l]:old.list_shared_begin[l] + sc]
            b = new.ids[new.list_shared_begin[l]:new.list_shared_begin[l] + sc]
            assert (a == b).all()
            rc = int(old.list_ref_cnt[l])
            ro, rn = int(old.list_ref_begin[l]), int(new.list_ref_begin[l])
            assert (old.ref_owner[ro:ro + rc] == new.ref_owner[rn:rn + rc]).all()
            assert (old.ref_nblocks[ro:ro + rc] == new.ref_nblocks[rn:rn + rc]).all()
            for r in range(rc):      # each old entry still names the same blocks' contents
                nb = int(old.ref_nblocks[ro + r])
                x = old.ids[old.ref_block_begin[ro + r]:old.ref_block_begin[ro + r] + nb]
                y = new.ids[new.ref_block_begin[rn + r]:new.ref_block_begin[rn + r] + nb]
                assert (x == y).all()
            grew += int(new.list_ref_cnt[l]) - rc
            # old miscellaneous items keep their places; new ones follow directly
            om = old.ids[old.list_misc_begin[l]:old.list_misc_begin[l] + old.list_misc_cnt[l]].reshape(-1)
            nm = new.ids[new.list_misc_begin[l]:new.list_misc_begin[l] + new.list_misc_cnt[l]].reshape(-1)
            k = int((om >= 0).sum())
            assert (nm[:k] == om[:k]).all()
            assert (nm[k:][nm[k:] >= 0] >= old.ntotal).all()
        assert grew > 0
        # a list may now hold two entries to the same owner
    owners = [tuple(h2.ref_owner[h2.list_ref_begin[l]:h2.list_ref_begin[l] + h2.list_ref_cnt[l]])
              for l in range(h2.nlist)]
    assert any(len(o) != len(set(o)) for o in owners)


@pytest.mark.parametrize("strict", [True, False])
def test_delete_keeps_the_rules_and_the_candidate_set(strict):
    base, steps = three_batches(23, True, strict)
    hx = steps[-1]
    g = np.random.Generator(np.random.PCG64(5))
    gone = g.choice(hx.ntotal, size=700, replace=False)
    live = np.ones(hx.ntotal, dtype=bool)
    live[gone] = False
    hd = ib.delete_ids(hx, gone)
    check_structure(hd, live, shared_full=False)
    check_search(hd, base, live, True, 4)
    # shared blocks: invalidated in place, nothing else moves
    owner, is_misc = ib._block_owner(hx)
    sh = ~is_misc & (owner >= 0)
    before, after = hx.ids[sh], hd.ids[sh]
    dead = np.isin(before, gone)
    assert (after[dead] == -1).all() and (after[~dead] == before[~dead]).all()
    assert dead.any()
    assert (hd.codes[sh] == hx.codes[sh]).all()
    # and then a further batch on top of the holes
    more = clumped(77, 400, 16, True)
    h3 = ib.append_batch(hd, more, strict=strict)
    live3 = np.concatenate([live, np.ones(400, dtype=bool)])
    check_structure(h3, live3, shared_full=False)
    check_search(h3, np.concatenate([base, more]), live3, True, 5)


def test_delete_one_by_one_moves_the_last_item():
    base, steps = three_batches(24, False, True)
    hx = steps[0]
    # a list with a miscellaneous area of at least two items
    l = next(l for l in range(hx.nlist) if (hx.ids[hx.list_misc_begin[l]:hx.list_misc_begin[l]
                                                  + hx.list_misc_cnt[l]] >= 0).sum() >= 2)
    mb = int(hx.list_misc_begin[l])
    flat = hx.ids[mb:mb + hx.list_misc_cnt[l]].reshape(-1)
    n = int((flat >= 0).sum())
    first, last = int(flat[0]), int(flat[n - 1])
    hd = ib.delete_ids(hx, [first])
    flat2 = hd.ids[mb:mb + hd.list_misc_cnt[l]].reshape(-1)
    assert int(flat2[0]) == last                   # the last item took the freed place
    assert (flat2[1:n - 1] == flat[1:n - 1]).all() and (flat2[n - 1:] < 0).all()
    assert hd.other.reshape(-1)[mb * BLK] == hx.other.reshape(-1)[mb * BLK + n - 1]
    assert (hd.codes.reshape(-1, hx.M // 2)[mb * BLK] == hx.codes.reshape(-1, hx.M // 2)[mb * BLK + n - 1]).all()
    with pytest.raises(KeyError):
        ib.delete_ids(hd, [first])
    with pytest.raises(KeyError):
        ib.delete_ids(hd, [hx.ntotal])
    # deleting the moved item afterwards finds it at its new place
    live = np.ones(hx.ntotal, dtype=bool)
    live[[first, last]] = False
    h2 = ib.delete_ids(hx, [first, last])
    check_structure(h2, live, shared_full=False)


def test_delete_everything():
    base, steps = three_batches(25, False, True)
    hx = steps[1]
    hd = ib.delete_ids(hx, np.arange(hx.ntotal)[::-1])
    assert (hd.ids == -1).all() and (hd.list_misc_cnt == 0).all()
    ox = oracle.OracleIndex(hd)
    r = oracle.search(ox, queries(1, 5, hx.d), 10, 4, 40)
    assert (r.ids == -1).all() and (r.cand_ids == -1).all() and (r.dco == 0).all()
