"""Host index construction (Alg. 1, 3, 4) against what the paper fixes about it."""
import numpy as np
import pytest

from paper_2601_07183_amd import datagen, index_build as ib


def _direct_nearest(x, c):
    d2 = ((x[:, None, :].astype(np.float64) - c[None].astype(np.float64)) ** 2).sum(-1)
    return np.argsort(d2, axis=1, kind="stable"), d2


def test_air_lambda_zero_is_second_nearest():
    # Section 4.1: with lambda = 0 AIR degenerates to choosing the second nearest list.
    x = datagen.random_vectors(1, 500, 8)
    c = datagen.random_vectors(2, 20, 8)
    a = ib.rair_assign(x, c, lam=0.0, n_cands=10, strict=True)
    order, _ = _direct_nearest(x, c)
    want = np.sort(order[:, :2], axis=1)
    assert (a == want).all()
    assert (a[:, 0] <= a[:, 1]).all()                     # Alg. 3 returns the pair ordered


def test_air_loss_of_primary_list():
    # Section 4.2: the loss of the primary list itself is (1 + lambda) ||r||^2.
    x = datagen.random_vectors(3, 50, 6)
    c = datagen.random_vectors(4, 12, 6)
    order, d2 = _direct_nearest(x, c)
    cand = order[:, :5]
    for lam in (0.0, 0.5, 2.0):
        loss = ib.air_loss(x, c[cand], lam)
        r0 = np.take_along_axis(d2, cand[:, :1], 1)[:, 0]
        assert np.allclose(loss[:, 0], (1 + lam) * r0, rtol=1e-12)
        # the general entry, written out independently: ||c' - x||^2 + lam (c - x).(c' - x)
        for i in range(0, 50, 7):
            for j in range(5):
                r = c[cand[i, 0]].astype(np.float64) - x[i]
                rp = c[cand[i, j]].astype(np.float64) - x[i]
                assert np.isclose(loss[i, j], rp @ rp + lam * (r @ rp), rtol=1e-12)


def test_nonstrict_single_assignment_condition():
    # RAIR stores a vector once iff no candidate list beats (1 + lambda) ||r||^2 (Section 4.2).
    x = datagen.random_vectors(5, 800, 4)
    c = datagen.random_vectors(6, 16, 4)
    lam = 0.5
    a = ib.rair_assign(x, c, lam=lam, n_cands=16, strict=False)
    order, d2 = _direct_nearest(x, c)
    loss = ib.air_loss(x, c[order], lam)
    single = (loss[:, 1:] >= loss[:, :1]).all(1)
    assert ((a[:, 0] == a[:, 1]) == single).all()
    assert single.any() and (~single).any()
    # strict mode never stores a vector once
    s = ib.rair_assign(x, c, lam=lam, n_cands=16, strict=True)
    assert (s[:, 0] < s[:, 1]).all()
    # and the primary list is always one of the pair
    assert ((a[:, 0] == order[:, 0]) | (a[:, 1] == order[:, 0])).all()


def test_air_prefers_opposite_residual():
    # Fig. 2 of the paper in numbers: x at the origin, primary centroid at +1 on the first axis,
    # two other centroids at equal distance 1.5, one on the same side, one on the opposite side.
    x = np.zeros((1, 2), dtype=np.float32)
    c = np.array([[1.0, 0.0], [1.5, 0.0], [-1.5, 0.0], [0.0, 1.5]], dtype=np.float32)
    a = ib.rair_assign(x, c, lam=0.5, n_cands=4, strict=True)
    assert a.tolist() == [[0, 2]]
    a0 = ib.rair_assign(x, c, lam=0.0, n_cands=4, strict=True)
    assert a0.tolist() == [[0, 1]]                        # ties on distance go to the lower id


def test_seil_layout_worked_example():
    # Alg. 4 by hand: 3 lists.  cell(0,1): 70 items -> 2 full blocks in list 0 + 6 leftovers in
    # the misc areas of lists 0 and 1; cell(0,0): 5 items -> misc of list 0 only;
    # cell(1,2): 33 items -> 1 block in list 1 + 1 leftover in lists 1 and 2.
    assign = np.array([[0, 1]] * 70 + [[0, 0]] * 5 + [[1, 2]] * 33, dtype=np.int32)
    n = assign.shape[0]
    perm = np.random.Generator(np.random.PCG64(7)).permutation(n)
    assign = assign[perm]
    ids = np.arange(n, dtype=np.int64)
    codes = (np.arange(n, dtype=np.uint8)[:, None] + np.zeros((1, 2), dtype=np.uint8))
    lay = ib.seil_insert(assign, codes, ids, 3)
    assert lay["list_shared_cnt"].tolist() == [2, 1, 0]
    assert lay["list_misc_cnt"].tolist() == [1, 1, 1]      # 5+6=11, 6+1=7, 1 items
    assert lay["list_shared_begin"].tolist() == [0, 3, 5]
    assert lay["list_misc_begin"].tolist() == [2, 4, 5]
    assert lay["list_ref_cnt"].tolist() == [0, 1, 1]
    assert lay["ref_owner"].tolist() == [0, 1]
    assert lay["ref_block_begin"].tolist() == [0, 3]
    assert lay["ref_nblocks"].tolist() == [2, 1]
    in01 = np.sort(np.flatnonzero((assign == [0, 1]).all(1)))
    in00 = np.sort(np.flatnonzero((assign == [0, 0]).all(1)))
    in12 = np.sort(np.flatnonzero((assign == [1, 2]).all(1)))
    # sort key is {list1, list2, id}: blocks hold the cell's ids in increasing order
    assert lay["ids"][0].tolist() == in01[:32].tolist()
    assert lay["ids"][1].tolist() == in01[32:64].tolist()
    # list 0 misc: cell (0,0) comes before (0,1) in the sorted order
    assert lay["ids"][2][:11].tolist() == in00.tolist() + in01[64:].tolist()
    assert lay["other"][2][:11].tolist() == [0] * 5 + [1] * 6
    assert (lay["ids"][2][11:] == -1).all() and (lay["other"][2][11:] == -1).all()
    assert lay["ids"][3].tolist() == in12[:32].tolist()
    # list 1 misc: leftovers of (0,1) tagged 0, then of (1,2) tagged 2
    assert lay["ids"][4][:7].tolist() == in01[64:].tolist() + in12[32:].tolist()
    assert lay["other"][4][:7].tolist() == [0] * 6 + [2]
    assert lay["ids"][5][:1].tolist() == in12[32:].tolist()
    assert lay["other"][5][:1].tolist() == [1]
    assert (lay["other"][[0, 1, 3]] == -1).all()
    # codes travel with their ids
    valid = lay["ids"] >= 0
    assert (lay["codes"][valid][:, 0] == lay["ids"][valid].astype(np.uint8)).all()


def _check_layout(hx):
    n, nlist, B = hx.ntotal, hx.nlist, hx.blk
    a = hx.assign.astype(np.int64)
    key = a[:, 0] * nlist + a[:, 1]
    cells, cnt = np.unique(key, return_counts=True)
    c1, c2 = cells // nlist, cells % nlist
    nb, nm = cnt // B, cnt % B
    # count conservation (Alg. 4 pass 1)
    assert (hx.list_shared_cnt == np.bincount(c1, weights=nb, minlength=nlist)).all()
    misc_items = np.bincount(c1, weights=nm, minlength=nlist) + \
        np.bincount(c2[c1 != c2], weights=nm[c1 != c2], minlength=nlist)
    assert (hx.list_misc_cnt == (misc_items + B - 1) // B).all()
    slots = (hx.ids >= 0).sum()
    assert slots == (B * nb).sum() + (np.where(c1 != c2, 2, 1) * nm).sum()
    # only the last misc block of a list may be partly filled; shared blocks are full
    for L in range(nlist):
        sb, sc = hx.list_shared_begin[L], hx.list_shared_cnt[L]
        mb, mc = hx.list_misc_begin[L], hx.list_misc_cnt[L]
        assert mb == sb + sc
        assert (hx.ids[sb:sb + sc] >= 0).all()
        assert (hx.other[sb:sb + sc] == -1).all()
        if mc:
            assert (hx.ids[mb:mb + mc - 1] >= 0).all()
            fill = (hx.ids[mb + mc - 1] >= 0)
            assert fill[0] and (np.diff(fill.astype(int)) <= 0).all()
            assert fill.sum() == misc_items[L] - B * (mc - 1)
        # members of a shared block all belong to one cell (L, j)
        for b in range(sb, sb + sc):
            v = hx.ids[b]
            assert (a[v, 0] == L).all() and (a[v, 1] == a[v[0], 1]).all()
        # misc items: tag = the other list of the item's pair
        for b in range(mb, mb + mc):
            ok = hx.ids[b] >= 0
            v, t = hx.ids[b][ok], hx.other[b][ok]
            assert (((a[v, 0] == L) & (a[v, 1] == t)) | ((a[v, 1] == L) & (a[v, 0] == t))).all()
        # reference entries of L point into their owner's shared area at that cell's blocks
        for r in range(hx.list_ref_begin[L], hx.list_ref_begin[L] + hx.list_ref_cnt[L]):
            o, bb, nbk = hx.ref_owner[r], hx.ref_block_begin[r], hx.ref_nblocks[r]
            assert o < L and nbk >= 1
            assert hx.list_shared_begin[o] <= bb and bb + nbk <= hx.list_shared_begin[o] + hx.list_shared_cnt[o]
            v = hx.ids[bb:bb + nbk].ravel()
            assert (a[v, 0] == o).all() and (a[v, 1] == L).all()
            assert nbk == cnt[(c1 == o) & (c2 == L)][0] // B
    # one reference entry per two-list cell with at least one full block
    assert hx.nrefs == ((c1 != c2) & (nb > 0)).sum()
    # every vector: once in a shared block, or once in the misc area of each of its lists
    occ = np.bincount(hx.ids[hx.ids >= 0], minlength=n)
    shared_mask = np.zeros(hx.nblocks, dtype=bool)
    for L in range(nlist):
        shared_mask[hx.list_shared_begin[L]:hx.list_shared_begin[L] + hx.list_shared_cnt[L]] = True
    in_shared = np.bincount(hx.ids[shared_mask].ravel(), minlength=n)
    assert set(np.unique(in_shared)) <= {0, 1}
    want = np.where(in_shared == 1, 1, np.where(a[:, 0] != a[:, 1], 2, 1))
    assert (occ == want).all()
    # codes stored with an item are that vector's codes
    valid = hx.ids >= 0
    assert (hx.codes[valid] == hx.vec_codes[hx.ids[valid]]).all()
    assert (hx.codes[~valid] == 0).all()


def test_seil_layout_invariants(small_index, small_index_nonstrict):
    _check_layout(small_index[1])
    _check_layout(small_index_nonstrict[1])
    hx = small_index_nonstrict[1]
    assert (hx.assign[:, 0] == hx.assign[:, 1]).any()      # cell (i,i) is exercised


def test_seil_layout_adversarial():
    x = datagen.random_vectors(21, 700, 8)
    cents = ib.kmeans(x, 8, 5, 1)
    cb = ib.train_pq(x, 4, 5, 2)
    g = np.random.Generator(np.random.PCG64(5))
    one_cell = np.tile(np.array([[2, 5]], dtype=np.int32), (700, 1))
    pairs = np.sort(g.integers(0, 8, size=(700, 2)), axis=1).astype(np.int32)
    tiny_cells = np.array([[i % 8, (i // 8) % 8] for i in range(700)], dtype=np.int32)
    tiny_cells = np.sort(tiny_cells, axis=1)[:300]
    for asg, xs in ((one_cell, x), (pairs, x), (tiny_cells, x[:300])):
        _check_layout(ib.add_vectors(xs, cents, cb, assign=asg))


def test_naive_layout_bytes_match_table4_accounting():
    # Table 4: single assignment costs N * (M/2 + 8) bytes (32 B codes + 8 B id per item for
    # M = 64); assigning every vector twice without SEIL costs exactly twice that.
    n, M = 1_000_000, 64
    assert n * (M // 2 + 8) == 40_000_000                   # 38.2 MiB
    assert abs(n * (M // 2 + 8) / 2 ** 20 - 38.2) < 0.06


def test_pq_encode_is_nearest_codeword(small_index):
    base, hx = small_index
    dsub = hx.d // hx.M
    sub = base.reshape(-1, hx.M, dsub).astype(np.float64)
    d2 = ((sub[:, :, None, :] - hx.codebook[None].astype(np.float64)) ** 2).sum(-1)
    code = d2.argmin(-1)
    lo, hi = hx.vec_codes & 15, hx.vec_codes >> 4
    best = d2.min(-1)
    got = np.empty_like(code)
    got[:, 0::2], got[:, 1::2] = lo, hi
    chosen = np.take_along_axis(d2, got[:, :, None], 2)[:, :, 0]
    assert np.allclose(chosen, best, rtol=1e-5, atol=1e-7)
    assert (got == code).mean() > 0.999


@pytest.mark.parametrize("blk", [16, 64])
def test_seil_layout_with_other_block_sizes(blk):
    # BLK_SZ of Alg. 4 is a parameter (Section 6.4 varies it): the same structural rules at 16 and 64
    x = datagen.random_vectors(21, 2500, 8)
    cents = ib.kmeans(x, 8, 5, 1)
    cb = ib.train_pq(x, 4, 5, 2)
    g = np.random.Generator(np.random.PCG64(5))
    pairs = np.sort(g.integers(0, 8, size=(2500, 2)), axis=1).astype(np.int32)
    hx = ib.add_vectors(x, cents, cb, assign=pairs, blk=blk)
    assert hx.blk == blk and hx.ids.shape[1] == blk and hx.nrefs > 0
    _check_layout(hx)
    _check_layout(ib.add_vectors(x, cents, cb, blk=blk))
    # a larger block stores fewer vectors once: the shared fraction shrinks with BLK_SZ
    shared = [ib.add_vectors(x, cents, cb, assign=pairs, blk=b).list_shared_cnt.sum() * b for b in (16, 32, 64)]
    assert shared[0] >= shared[1] >= shared[2]


def test_soar_lambda_zero_is_second_nearest_and_prefers_orthogonal_residuals():
    # Section 2.3 / Table 1: SOAR's loss is ||r'||^2 + lam (r.r' / ||r||)^2.  lam = 0 leaves the
    # second-nearest list; with lam > 0 a candidate whose residual is orthogonal to the first
    # one wins over a slightly nearer one whose residual is parallel to it.
    x = datagen.random_vectors(41, 400, 6)
    cents = datagen.random_vectors(42, 12, 6)
    d2 = ((x[:, None, :].astype(np.float64) - cents[None].astype(np.float64)) ** 2).sum(-1)
    two = np.sort(np.argsort(d2, axis=1, kind="stable")[:, :2], axis=1)
    assert (ib.soar_assign(x, cents, lam=0.0, n_cands=12) == two).all()
    # hand-worked: v at the origin, primary centroid at (1, 0) so r = (-1, 0); candidates
    # c_par = (-1.1, 0) (r' = (1.1, 0): parallel, ||r'||^2 = 1.21, projection^2 = 1.21) and
    # c_orth = (0, 1.2) (r' = (0, -1.2): orthogonal, ||r'||^2 = 1.44, projection 0)
    v = np.zeros((1, 2), dtype=np.float32)
    c = np.array([[1.0, 0.0], [-1.1, 0.0], [0.0, 1.2]], dtype=np.float32)
    assert ib.soar_assign(v, c, lam=0.0, n_cands=3).tolist() == [[0, 1]]
    assert ib.soar_assign(v, c, lam=1.0, n_cands=3).tolist() == [[0, 2]]       # 1.21 + 1.21 > 1.44
    loss = ib.soar_loss(v, c[None], 1.0)[0]
    assert np.allclose(loss, [1.0 + 1.0, 1.21 + 1.21, 1.44])
    # AIR on the same picture prefers the opposite residual instead (Table 1's contrast)
    assert ib.rair_assign(v, c, lam=0.5, n_cands=3).tolist() == [[0, 1]]


def test_save_and_load_index_round_trip(tmp_path):
    import dataclasses
    w = datagen.scaled(datagen.WORKLOADS["tiny"], 3000, nq=8, nlist=16)
    hx = ib.build_index(datagen.make_base(w), w.nlist, w.M, seed=w.seed, coarse_iters=3, pq_iters=3)
    path = str(tmp_path / "ix.npz")
    ib.save_index(hx, path)
    back = ib.load_index(path)
    for f in dataclasses.fields(hx):
        a, b = getattr(hx, f.name), getattr(back, f.name)
        if isinstance(a, np.ndarray):
            assert a.dtype == b.dtype and np.array_equal(a, b), f.name
        else:
            assert a == b, f.name
