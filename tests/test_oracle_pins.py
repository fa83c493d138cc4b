"""Pins of the CPU oracle against things other than itself: brute force, closed forms,
invariants stated by the paper, integer arithmetic.  No GPU."""
import numpy as np
import pytest

from oracle import oracle
from paper_2601_07183_amd import datagen, index_build as ib

from conftest import small_queries


def _exact_knn(q, base, k):
    """Textbook kNN in float64, ties by smaller id."""
    d2 = ((q[:, None, :].astype(np.float64) - base[None].astype(np.float64)) ** 2).sum(-1)
    order = np.lexsort((np.broadcast_to(np.arange(base.shape[0]), d2.shape), d2), axis=1)
    return order[:, :k], np.take_along_axis(d2, order[:, :k], 1)


# --- exact distance ------------------------------------------------------------------------

@pytest.mark.parametrize("d", [1, 2, 31, 32, 63, 64, 65, 96, 128, 200, 960])
def test_l2sqr_against_float64(d):
    a = datagen.random_vectors(d, 4, d, -3, 3)
    b = datagen.random_vectors(d + 1, 4, d, -3, 3)
    for i in range(4):
        want = ((a[i].astype(np.float64) - b[i].astype(np.float64)) ** 2).sum()
        got = oracle.l2sqr(a[i], b[i])
        assert abs(got - want) <= 1e-6 * want + 1e-30      # fp32 tree sum, d <= 960


def test_l2sqr_summation_order_is_the_stated_tree():
    # 64 interleaved partial sums, then p[j] += p[j^32], ^16, ... -- rebuilt here with numpy
    # float32 scalars; a different order changes low bits on this input.
    d = 200
    a = (datagen.random_vectors(5, 1, d, -1, 1)[0] * np.float32(1000.123)).astype(np.float32)
    b = datagen.random_vectors(6, 1, d, -1, 1)[0]
    p = np.zeros(64, dtype=np.float32)
    for i in range(d):
        diff = np.float32(a[i] - b[i])
        p[i % 64] = np.float32(p[i % 64] + np.float32(diff * diff))
    for s in (32, 16, 8, 4, 2, 1):
        p = (p + p[np.arange(64) ^ s]).astype(np.float32)
    assert oracle.l2sqr(a, b) == float(p[0])
    seq = np.float32(0)
    for i in range(d):
        diff = np.float32(a[i] - b[i])
        seq = np.float32(seq + np.float32(diff * diff))
    assert float(seq) != float(p[0])


def test_l2sqr_integer_data_is_exact_and_u8_agrees():
    g = np.random.Generator(np.random.PCG64(3))
    a = g.integers(0, 256, size=128).astype(np.float32)
    b8 = g.integers(0, 256, size=128).astype(np.uint8)
    want = int(((a.astype(np.int64) - b8.astype(np.int64)) ** 2).sum())
    assert want < 2 ** 24
    assert oracle.l2sqr(a, b8.astype(np.float32)) == want
    assert oracle.l2sqr(a, b8) == want


# --- coarse quantizer ----------------------------------------------------------------------

def test_coarse_is_the_nprobe_nearest_by_distance_then_id(small_index_int):
    base, hx = small_index_int
    ox = oracle.OracleIndex(hx)
    q = small_queries(1, 20, hx.d, integer=True)
    # make two centroids identical so that a distance tie exists
    hx2 = ib.add_vectors(base, np.vstack([hx.centroids[:-1], hx.centroids[:1]]), hx.codebook)
    ox2 = oracle.OracleIndex(hx2)
    for o, cents in ((ox, hx.centroids), (ox2, hx2.centroids)):
        d2 = ((q[:, None, :].astype(np.float64) - cents[None].astype(np.float64)) ** 2).sum(-1)
        for i in range(len(q)):
            lists, dists = oracle.coarse(o, q[i], 5)
            order = np.lexsort((np.arange(hx.nlist), d2[i].astype(np.float32)))
            assert np.allclose(dists, d2[i][lists], rtol=1e-6)
            assert (np.diff(dists) >= 0).all()
            got = set(lists.tolist())
            # float64 order can only differ from the fp32 one inside fp32 rounding
            kth = np.sort(d2[i])[4]
            assert all(d2[i][l] <= kth * (1 + 1e-6) for l in got)
    lists, dists = oracle.coarse(ox2, q[0], hx.nlist)
    pos0, posl = list(lists).index(0), list(lists).index(hx.nlist - 1)
    assert posl == pos0 + 1 and dists[pos0] == dists[posl]   # equal distance: smaller id first


# --- lookup table --------------------------------------------------------------------------

def test_lut_pq_identity(small_index):
    # Section 2.2: summing the table entries selected by a code gives the squared distance
    # between the query and the decoded vector.
    base, hx = small_index
    ox = oracle.OracleIndex(hx)
    q = small_queries(2, 8, hx.d)
    dsub = hx.d // hx.M
    code = np.empty((hx.ntotal, hx.M), dtype=np.int64)
    code[:, 0::2], code[:, 1::2] = hx.vec_codes & 15, hx.vec_codes >> 4
    decoded = hx.codebook[np.arange(hx.M)[None, :], code].reshape(hx.ntotal, hx.M * dsub)
    for i in range(len(q)):
        T, u8, bias, scale = oracle.lut(ox, q[i])
        est = T[np.arange(hx.M)[None, :], code[:200]].astype(np.float64).sum(1)
        want = ((q[i].astype(np.float64) - decoded[:200].astype(np.float64)) ** 2).sum(1)
        assert np.allclose(est, want, rtol=1e-5, atol=1e-6)


def test_lut_quantisation_bound_and_range(small_index):
    base, hx = small_index
    ox = oracle.OracleIndex(hx)
    q = small_queries(3, 8, hx.d)
    code = np.empty((hx.ntotal, hx.M), dtype=np.int64)
    code[:, 0::2], code[:, 1::2] = hx.vec_codes & 15, hx.vec_codes >> 4
    for i in range(len(q)):
        T, u8, bias, scale = oracle.lut(ox, q[i])
        assert (u8.min(1) == 0).all()                       # each row's minimum maps to 0
        assert u8.max() == 255                              # the widest row reaches 255
        span = (T.max(1) - T.min(1)).max()
        assert np.isclose(scale, 255.0 / span, rtol=1e-6)
        assert np.isclose(bias, T.min(1).astype(np.float64).sum(), rtol=1e-5)
        acc = u8[np.arange(hx.M)[None, :], code[:500]].astype(np.int64).sum(1)
        est = T[np.arange(hx.M)[None, :], code[:500]].astype(np.float64).sum(1)
        err = np.abs(bias + acc / scale - est)
        assert (err <= hx.M / (2 * scale) * (1 + 1e-4) + 1e-5 * est).all()
        # rounding is to nearest: every entry within half a step
        step = (T - T.min(1, keepdims=True)).astype(np.float64) * scale
        assert (np.abs(step - u8) <= 0.5 + 1e-3).all()


def test_lut_rounds_half_to_even():
    # One worked table: M = 2, dsub = 1, query 0.  Codewords sqrt(t) give T = t exactly for the
    # chosen t; the widest row spans 510, so s = 0.5 and (T - b) * s hits .5 cases.
    class H:
        pass
    t0 = np.array([0, 1, 3, 5, 7, 9, 11, 510, 2, 4, 6, 8, 10, 12, 14, 16], dtype=np.float64)
    t1 = np.array([4, 5, 7, 9, 11, 13, 15, 17, 19, 21, 23, 25, 27, 29, 31, 33], dtype=np.float64)
    cb = np.sqrt(np.stack([t0, t1]))[:, :, None].astype(np.float32)
    T_exact = (cb[:, :, 0].astype(np.float32) ** 2).astype(np.float32)
    base = np.zeros((4, 2), dtype=np.float32)
    hx = ib.add_vectors(base, np.zeros((2, 2), dtype=np.float32), cb,
                        assign=np.array([[0, 1]] * 4, dtype=np.int32))
    T, u8, bias, scale = oracle.lut(oracle.OracleIndex(hx), np.zeros(2, dtype=np.float32))
    assert (T == T_exact).all()
    # only check entries whose fp32 square is the exact integer (sqrt rounding may break some)
    ok = T_exact == np.stack([t0, t1])
    assert ok[0, [0, 1, 2, 3, 7]].all() and ok[1, 0]
    assert scale == 0.5 and bias == float(T_exact[0].min() + T_exact[1].min())
    want0 = {0: 0, 1: 0, 3: 2, 5: 2, 7: 4, 9: 4, 11: 6, 510: 255}   # x.5 goes to the even integer
    for c in range(16):
        if ok[0, c] and int(t0[c]) in want0:
            assert u8[0, c] == want0[int(t0[c])]
    # second row: (T - 4) * 0.5 = 0, .5, 1.5, 2.5, ... -> 0, 0, 2, 2, 4, 4, ...
    for c in range(16):
        if ok[1, c]:
            x = (t1[c] - 4) * 0.5
            assert u8[1, c] == int(np.rint(x))


# --- whole path ----------------------------------------------------------------------------

def test_brute_force_knn_when_everything_is_probed_and_refined(small_index_int):
    # nprobe = nlist and bigK >= N: the path must return the exact kNN (recall 1).  Integer data
    # makes every distance exact, so ids match including ties.
    base, hx = small_index_int
    ox = oracle.OracleIndex(hx)
    q = small_queries(4, 25, hx.d, integer=True)
    want_ids, want_d = _exact_knn(q, base, 10)
    for layout in ("seil", "naive"):
        r = oracle.search(ox, q, 10, hx.nlist, hx.ntotal, layout=layout)
        assert (r.ids == want_ids).all()
        assert (r.dists.astype(np.float64) == want_d).all()


def test_brute_force_knn_float_data(small_index):
    base, hx = small_index
    ox = oracle.OracleIndex(hx)
    q = small_queries(5, 25, hx.d)
    want_ids, want_d = _exact_knn(q, base, 10)
    r = oracle.search(ox, q, 10, hx.nlist, hx.ntotal)
    assert np.allclose(r.dists, want_d, rtol=1e-5)
    assert (r.ids == want_ids).mean() > 0.99               # only fp32 near-ties may swap
    for i in range(len(q)):
        assert set(r.ids[i]) == set(want_ids[i]) or \
            np.allclose(np.sort(r.dists[i]), want_d[i], rtol=1e-5)


def test_candidates_are_the_smallest_scores_by_definition(small_index):
    # Independent numpy evaluation of steps 2-4 of the definition from the per-vector view.
    base, hx = small_index
    ox = oracle.OracleIndex(hx)
    q = small_queries(6, 10, hx.d)
    code = np.empty((hx.ntotal, hx.M), dtype=np.int64)
    code[:, 0::2], code[:, 1::2] = hx.vec_codes & 15, hx.vec_codes >> 4
    for nprobe in (1, 3, 7, hx.nlist):
        r = oracle.search(ox, q, 5, nprobe, 50)
        for i in range(len(q)):
            probed = np.zeros(hx.nlist, dtype=bool)
            probed[r.probes[i]] = True
            member = probed[hx.assign[:, 0]] | probed[hx.assign[:, 1]]
            acc = r.lut[i][np.arange(hx.M)[None, :], code].astype(np.int64).sum(1)
            ids = np.flatnonzero(member)
            order = ids[np.lexsort((ids, acc[ids]))][:50]
            n = len(order)
            assert (r.cand_ids[i][:n] == order).all() and (r.cand_ids[i][n:] == -1).all()
            assert (r.cand_acc[i][:n] == acc[order]).all()
            # refine: exact distances of the candidates, K smallest by (distance, id)
            d2 = np.array([oracle.l2sqr(q[i], base[v]) for v in order], dtype=np.float32)
            top = order[np.lexsort((order, d2))][:5]
            assert (r.ids[i][:len(top)] == top).all()


@pytest.mark.parametrize("which", ["strict", "nonstrict", "int"])
def test_seil_equals_naive_layout(which, small_index, small_index_nonstrict, small_index_int):
    base, hx = {"strict": small_index, "nonstrict": small_index_nonstrict,
                "int": small_index_int}[which]
    ox = oracle.OracleIndex(hx)
    q = small_queries(7, 40, hx.d, integer=(which == "int"))
    for nprobe in (1, 2, 5, 11, hx.nlist):
        a = oracle.search(ox, q, 10, nprobe, 60, layout="seil")
        b = oracle.search(ox, q, 10, nprobe, 60, layout="naive")
        assert (a.cand_ids == b.cand_ids).all() and (a.cand_acc == b.cand_acc).all()
        assert (a.ids == b.ids).all() and (a.dists == b.dists).all()


def test_seil_equals_naive_on_adversarial_assignments():
    x = datagen.random_vectors(31, 900, 8)
    q = datagen.random_vectors(32, 30, 8)
    cents = ib.kmeans(x, 8, 5, 1)
    cb = ib.train_pq(x, 4, 5, 2)
    g = np.random.Generator(np.random.PCG64(9))
    cases = [
        np.tile(np.array([[2, 5]], dtype=np.int32), (900, 1)),                # one huge cell
        np.sort(g.integers(0, 8, size=(900, 2)), axis=1).astype(np.int32),     # random pairs
        np.sort(np.array([[i % 8, (i // 8) % 8] for i in range(900)]), axis=1)[:300].astype(np.int32),
        np.tile(np.array([[3, 3]], dtype=np.int32), (900, 1)),                # all single-assigned
    ]
    for asg in cases:
        hx = ib.add_vectors(x[:len(asg)], cents, cb, assign=asg)
        ox = oracle.OracleIndex(hx)
        for nprobe in (1, 2, 4, 8):
            a = oracle.search(ox, q, 5, nprobe, 40, layout="seil", trace=True)
            b = oracle.search(ox, q, 5, nprobe, 40, layout="naive")
            assert (a.cand_ids == b.cand_ids).all() and (a.ids == b.ids).all()
            assert a.push_count.max() <= 1 and a.block_count.max() <= 1


def test_each_vector_pushed_at_most_once_and_dco_identity(small_index, small_index_nonstrict):
    for base, hx in (small_index, small_index_nonstrict):
        ox = oracle.OracleIndex(hx)
        q = small_queries(8, 30, hx.d)
        a = hx.assign.astype(np.int64)
        key = a[:, 0] * hx.nlist + a[:, 1]
        cells, cnt = np.unique(key, return_counts=True)
        c1, c2 = cells // hx.nlist, cells % hx.nlist
        members = np.bincount(a[:, 0], minlength=hx.nlist) + \
            np.bincount(a[:, 1][a[:, 0] != a[:, 1]], minlength=hx.nlist)
        for nprobe in (1, 4, 9, hx.nlist):
            r = oracle.search(ox, q, 10, nprobe, 50, trace=True)
            assert r.push_count.max() <= 1                  # no id enters the queue twice
            assert r.block_count.max() <= 1                 # no block is scored twice
            for i in range(len(q)):
                probed = np.zeros(hx.nlist, dtype=bool)
                probed[r.probes[i]] = True
                member = probed[a[:, 0]] | probed[a[:, 1]]
                assert ((r.push_count[i] == 1) == member).all()
                # cost analysis of Section 5.2: n_vec_selected - n_vec_shared
                both = probed[c1] & probed[c2] & (c1 != c2)
                want = members[probed].sum() - 32 * (cnt[both] // 32).sum()
                assert r.dco[i] == want
            if nprobe == hx.nlist:
                assert (r.push_count == 1).all()


def test_queries_are_independent(small_index):
    # Alg. 2 keeps no state across queries: permuting or splitting the batch permutes or splits
    # the output.
    base, hx = small_index
    ox = oracle.OracleIndex(hx)
    q = small_queries(9, 24, hx.d)
    r = oracle.search(ox, q, 10, 4, 40)
    perm = np.random.Generator(np.random.PCG64(1)).permutation(len(q))
    rp = oracle.search(ox, q[perm], 10, 4, 40)
    assert (rp.ids == r.ids[perm]).all() and (rp.dists == r.dists[perm]).all()
    r1 = oracle.search(ox, q[:7], 10, 4, 40, nthreads=1)
    assert (r1.ids == r.ids[:7]).all()


def test_short_lists_are_padded(small_index):
    base, hx = small_index
    ox = oracle.OracleIndex(hx)
    q = small_queries(10, 5, hx.d)
    r = oracle.search(ox, q, 10, 1, hx.ntotal)              # bigK larger than any list
    n = (r.cand_ids >= 0).sum(1)
    assert (n < hx.ntotal).all() and (n >= 10).all()
    for i in range(len(q)):
        assert (r.cand_ids[i][n[i]:] == -1).all()
    with pytest.raises(ValueError):
        oracle.search(ox, q, 10, 0, 40)
    with pytest.raises(ValueError):
        oracle.search(ox, q, 50, 1, 40)


def test_tiny_workload_recall_is_monotone_and_layouts_agree(tiny_workload):
    w, base, q, hx = tiny_workload
    ox = oracle.OracleIndex(hx)
    gt, _ = _exact_knn(q[:60], base, w.k)
    last = -1.0
    for nprobe in w.nprobes:
        r = oracle.search(ox, q[:60], w.k, nprobe, w.refine_k)
        n = oracle.search(ox, q[:60], w.k, nprobe, w.refine_k, layout="naive")
        assert (r.ids == n.ids).all() and (r.cand_ids == n.cand_ids).all()
        rec = np.mean([len(set(r.ids[i]) & set(gt[i])) / w.k for i in range(60)])
        assert rec >= last - 0.02
        last = rec


# --- PQ encoding ---------------------------------------------------------------------------

def _unpack(codes, M):
    out = np.empty((codes.shape[0], M), dtype=np.int64)
    out[:, 0::2], out[:, 1::2] = codes & 15, codes >> 4
    return out


def test_pq_encode_is_the_nearest_codeword():
    # Alg. 1 / Section 2.2: against a float64 argmin wherever float64 separates the two best
    # codewords clearly; a transposed codebook axis, a swapped nibble or a wrong sub-vector
    # offset all fail here
    g = np.random.Generator(np.random.PCG64(5))
    for d, M in ((32, 16), (96, 48), (60, 6)):
        dsub = d // M
        cb = g.standard_normal((M, 16, dsub)).astype(np.float32)
        x = g.standard_normal((300, d)).astype(np.float32)
        got = _unpack(oracle.pq_encode(cb, x), M)
        d2 = ((x.reshape(300, M, 1, dsub).astype(np.float64) - cb[None].astype(np.float64)) ** 2).sum(-1)
        best = d2.argmin(-1)
        two = np.sort(d2, axis=-1)[..., :2]
        clear = two[..., 1] - two[..., 0] > 1e-5 * (1.0 + two[..., 1])
        assert clear.mean() > 0.99
        assert (got[clear] == best[clear]).all()
        # and where it is not clear, the chosen codeword is still a nearest one up to rounding
        chosen = np.take_along_axis(d2, got[..., None], -1)[..., 0]
        assert (chosen <= two[..., 0] + 1e-5 * (1.0 + two[..., 1])).all()


def test_pq_encode_codewords_encode_to_themselves_and_ties_take_the_first():
    g = np.random.Generator(np.random.PCG64(6))
    M, dsub = 8, 4
    cb = g.standard_normal((M, 16, dsub)).astype(np.float32)
    cb[:, 9] = cb[:, 3]                                   # codeword 9 duplicates codeword 3
    # vector j is made of codeword (j + m) % 16 of every sub-quantizer m
    pick = (np.arange(16)[:, None] + np.arange(M)[None, :]) % 16
    x = cb[np.arange(M)[None, :], pick].reshape(16, M * dsub)
    got = _unpack(oracle.pq_encode(cb, x), M)
    want = np.where(pick == 9, 3, pick)                   # distance 0 twice: the first wins
    assert (got == want).all()


def test_pq_encode_packing_matches_the_index_layout(small_index):
    # byte i of a code holds sub-quantizer 2i in the low nibble: re-encoding the base vectors with
    # the index's codebook gives codes whose decoded vectors are as close as the stored codes'
    base, hx = small_index
    dsub = hx.d // hx.M
    codes = oracle.pq_encode(hx.codebook, base[:500])
    def err(c):
        dec = hx.codebook[np.arange(hx.M)[None, :], _unpack(c, hx.M)].reshape(len(c), hx.M * dsub)
        return ((base[:len(c)].astype(np.float64) - dec) ** 2).sum(1)
    stored = hx.vec_codes[:500]
    assert np.allclose(err(codes), err(stored), rtol=1e-6, atol=1e-9)
    assert (codes == stored).mean() > 0.999               # the builder's own encoder, other arithmetic


# --- RairAssign ----------------------------------------------------------------------------

def _assign_float64(c, x, n_cands, lam, strict):
    """Alg. 3 written out in float64 numpy; also returns how clearly each decision is separated."""
    d2 = ((x[:, None, :].astype(np.float64) - c[None].astype(np.float64)) ** 2).sum(-1)
    order = np.argsort(d2, axis=1, kind="stable")
    n_cands = min(n_cands, c.shape[0])
    cand = order[:, :n_cands]
    srt = np.take_along_axis(d2, order, 1)
    gap_c = (srt[:, 1:n_cands + 1] - srt[:, :n_cands][:, : srt[:, 1:n_cands + 1].shape[1]]).min(1) if c.shape[0] > 1 else np.ones(len(x))
    r = c[cand].astype(np.float64) - x[:, None, :].astype(np.float64)
    loss = (r * r).sum(-1) + lam * (r * r[:, :1, :]).sum(-1)
    start = 1 if strict else 0
    if start >= n_cands:
        second, gap_l = cand[:, 0], np.ones(len(x))
    else:
        sub = loss[:, start:]
        pos = sub.argmin(1)
        second = cand[np.arange(len(x)), pos + start]
        two = np.sort(sub, axis=1)[:, :2]
        gap_l = two[:, 1] - two[:, 0] if sub.shape[1] > 1 else np.ones(len(x))
    first = cand[:, 0]
    pair = np.stack([np.minimum(first, second), np.maximum(first, second)], 1).astype(np.int32)
    return pair, (gap_c > 1e-4) & (gap_l > 1e-4)


@pytest.mark.parametrize("strict", [True, False])
@pytest.mark.parametrize("lam", [0.0, 0.5, 2.0])
def test_rair_assign_against_float64(strict, lam):
    g = np.random.Generator(np.random.PCG64(17))
    c = g.standard_normal((40, 24)).astype(np.float32)
    x = (c[g.integers(0, 40, 500)] + 0.7 * g.standard_normal((500, 24))).astype(np.float32)
    want, clear = _assign_float64(c, x, 10, lam, strict)
    got = oracle.rair_assign(c, x, 10, lam, strict)
    assert clear.mean() > 0.95
    assert (got[clear] == want[clear]).all()
    assert (got[:, 0] <= got[:, 1]).all()


def test_rair_assign_special_cases():
    g = np.random.Generator(np.random.PCG64(18))
    c = g.standard_normal((30, 16)).astype(np.float32)
    x = g.standard_normal((200, 16)).astype(np.float32)
    d2 = ((x[:, None, :].astype(np.float64) - c[None].astype(np.float64)) ** 2).sum(-1)
    near = np.argsort(d2, axis=1, kind="stable")
    # lambda = 0, strict: the loss is the distance, so the secondary list is the second nearest
    got = oracle.rair_assign(c, x, 10, 0.0, True)
    assert (np.sort(near[:, :2], axis=1) == got).all()
    # lambda = 0, not strict: the primary list minimises its own loss, the vector is stored once
    got = oracle.rair_assign(c, x, 10, 0.0, False)
    assert (got[:, 0] == near[:, 0]).all() and (got[:, 1] == near[:, 0]).all()
    # one candidate only: nothing to choose, also when strict
    got = oracle.rair_assign(c, x, 1, 0.5, True)
    assert (got[:, 0] == near[:, 0]).all() and (got[:, 1] == near[:, 0]).all()
    # more candidates asked for than lists: all lists are candidates
    assert (oracle.rair_assign(c, x, 100, 0.5, True) == oracle.rair_assign(c, x, 30, 0.5, True)).all()
    # hand-worked: v at the origin, c0 = (1, 0) nearest, c1 = (1.1, 0.1) on the same side, c2 =
    # (-1.5, 0) on the far side.  lambda = 0: second nearest (c1).  lambda = 1: loss1 = 1.22 + 1.1,
    # loss2 = 2.25 - 1.5, so the list on the far side wins -- the point of the AIR metric.
    c3 = np.array([[1.0, 0.0], [1.1, 0.1], [-1.5, 0.0]], dtype=np.float32)
    v0 = np.zeros((1, 2), dtype=np.float32)
    assert oracle.rair_assign(c3, v0, 3, 0.0, True).tolist() == [[0, 1]]
    assert oracle.rair_assign(c3, v0, 3, 1.0, True).tolist() == [[0, 2]]


def test_air_metric_ranks_like_the_loss_it_stands_for():
    # Section 4.2 defines the loss of a second centroid c' as the mean over queries q, uniform in
    # a ball around x, of ReLU(-cos(angle q x c)) * (|q - c'|^2 - |q - x|^2), and Theorem 1 replaces
    # it by |r'|^2 + lambda r.r' (r = c - x, r' = c' - x).  Here the mean is taken by Monte Carlo
    # from that definition (same queries for every c'), the two coefficients are fitted, and the
    # oracle's assignment at the fitted lambda has to pick the c' of least sampled loss.
    g = np.random.Generator(np.random.PCG64(31))
    d, nq = 6, 400000
    u = g.standard_normal((nq, d))
    u *= (g.uniform(0, 1, nq) ** (1.0 / d) / np.linalg.norm(u, axis=1))[:, None] * 1.5   # ball, radius 1.5
    for trial in range(6):
        x = g.standard_normal(d)
        r = g.standard_normal(d)
        r *= 1.0 / np.linalg.norm(r)                       # the nearest centroid, at distance 1
        others = g.standard_normal((9, d))
        others *= (g.uniform(1.05, 1.6, 9) / np.linalg.norm(others, axis=1))[:, None]
        others[0] = 1.06 * r + 0.02 * others[0]            # second nearest, on the same side as c
        rp = np.concatenate([r[None], others])             # candidates' residuals, nearest first
        w = np.maximum(0.0, -(u @ r) / (np.linalg.norm(u, axis=1) * np.linalg.norm(r)))
        gain = ((u[:, None, :] - rp[None, 1:, :]) ** 2).sum(-1) - (u * u).sum(-1)[:, None]
        loss_mc = (w[:, None] * gain).mean(0)              # [9] sampled loss of each second centroid
        feats = np.stack([(rp[1:] ** 2).sum(1), rp[1:] @ r], 1)
        (a, b), res, _, _ = np.linalg.lstsq(feats, loss_mc, rcond=None)
        assert a > 0 and b > 0                             # lambda = b / a > 0, as the theorem says
        # the sampled loss is the two-term form up to sampling noise (about nq ** -0.5)
        noise = np.abs(feats @ [a, b] - loss_mc).max()
        assert noise < 3e-3 * np.abs(loss_mc).max()
        lam = b / a
        cents = (x[None] + rp).astype(np.float32)
        got = oracle.rair_assign(cents, x[None].astype(np.float32), 10, float(lam), True)
        best = 1 + int(np.argmin(loss_mc))
        order = np.sort(loss_mc)
        assert order[1] - order[0] > 4 * noise             # a clear winner
        assert got.tolist() == [[0, best]]
        assert best != 1                                   # never the second nearest here: it lies on c's side


# --- inner-product metric (Section 6.4 applies SEIL to an inner-product index) --------------------

def _ip_index(seed, integer=False, n=3000, d=16, nlist=16, M=8, blk=32):
    base = datagen.random_vectors(seed, n, d)
    g = np.random.Generator(np.random.PCG64(seed + 99))
    centers = g.uniform(-1, 1, size=(8, d)).astype(np.float32)
    base = (centers[g.integers(0, 8, size=n)] + 0.25 * base).astype(np.float32)
    if integer:
        base = np.clip(np.rint(base * 60 + 128), 0, 255).astype(np.float32)
    return base, ib.build_index(base, nlist, M, seed=seed, coarse_iters=8, pq_iters=8, metric="ip",
                                lam=1.0, blk=blk)


@pytest.mark.parametrize("d", [1, 31, 64, 65, 128, 200, 960])
def test_ip_against_float64_and_the_stated_tree(d):
    a = (datagen.random_vectors(d, 3, d, -3, 3) * np.float32(17.25)).astype(np.float32)
    b = datagen.random_vectors(d + 1, 3, d, -3, 3)
    for i in range(3):
        want = (a[i].astype(np.float64) * b[i].astype(np.float64)).sum()
        got = oracle.ip(a[i], b[i])
        assert abs(got - want) <= 1e-6 * (np.abs(a[i].astype(np.float64) * b[i]).sum()) + 1e-30
        p = np.zeros(64, dtype=np.float32)
        for t in range(d):
            p[t % 64] = np.float32(p[t % 64] + np.float32(a[i][t] * b[i][t]))
        for s in (32, 16, 8, 4, 2, 1):
            p = (p + p[np.arange(64) ^ s]).astype(np.float32)
        assert got == float(p[0])
    g = np.random.Generator(np.random.PCG64(4))
    ai = g.integers(0, 256, size=128).astype(np.float32)
    b8 = g.integers(0, 256, size=128).astype(np.uint8)
    want = int((ai.astype(np.int64) * b8.astype(np.int64)).sum())
    assert want < 2 ** 24 and oracle.ip(ai, b8) == want and oracle.ip(ai, b8.astype(np.float32)) == want


def test_ip_coarse_is_the_nprobe_largest_products_then_id():
    base, hx = _ip_index(21, integer=True)
    q = small_queries(1, 20, hx.d, integer=True)
    hx2 = ib.add_vectors(base, np.vstack([hx.centroids[:-1], hx.centroids[:1]]), hx.codebook, metric="ip")
    for h in (hx, hx2):
        o = oracle.OracleIndex(h)
        assert o.metric == "ip"
        prod = q.astype(np.float64) @ h.centroids.astype(np.float64).T
        for i in range(len(q)):
            lists, dots = oracle.coarse(o, q[i], 5)
            assert np.allclose(dots, prod[i][lists], rtol=1e-6)
            assert (np.diff(dots) <= 0).all()                  # reported as products, largest first
            kth = np.sort(prod[i])[-5]
            assert all(prod[i][l] >= kth - 1e-6 * abs(kth) for l in lists)
    lists, dots = oracle.coarse(oracle.OracleIndex(hx2), q[0], hx.nlist)
    pos0, posl = list(lists).index(0), list(lists).index(hx.nlist - 1)
    assert posl == pos0 + 1 and dots[pos0] == dots[posl]       # equal product: smaller id first


def test_ip_lut_identity_and_quantisation():
    # the table entries selected by a code sum to minus the inner product with the decoded vector
    base, hx = _ip_index(22)
    ox = oracle.OracleIndex(hx)
    q = small_queries(2, 8, hx.d)
    dsub = hx.d // hx.M
    code = np.empty((hx.ntotal, hx.M), dtype=np.int64)
    code[:, 0::2], code[:, 1::2] = hx.vec_codes & 15, hx.vec_codes >> 4
    decoded = hx.codebook[np.arange(hx.M)[None, :], code].reshape(hx.ntotal, hx.M * dsub)
    for i in range(len(q)):
        T, u8, bias, scale = oracle.lut(ox, q[i])
        est = T[np.arange(hx.M)[None, :], code[:300]].astype(np.float64).sum(1)
        want = -(decoded[:300].astype(np.float64) @ q[i].astype(np.float64))
        assert np.allclose(est, want, rtol=1e-5, atol=1e-5)
        assert (u8.min(1) == 0).all() and u8.max() == 255
        span = (T.max(1) - T.min(1)).max()
        assert np.isclose(scale, 255.0 / span, rtol=1e-6)
        step = (T - T.min(1, keepdims=True)).astype(np.float64) * scale
        assert (np.abs(step - u8) <= 0.5 + 1e-3).all()


def test_ip_brute_force_when_everything_is_probed_and_refined():
    # integer data: every product sum is exact, ties are real and go to the smaller id
    base, hx = _ip_index(23, integer=True, n=1500)
    q = small_queries(9, 12, hx.d, integer=True)
    r = oracle.search(oracle.OracleIndex(hx), q, 10, hx.nlist, hx.ntotal)
    prod = q.astype(np.int64) @ base.astype(np.int64).T
    order = np.lexsort((np.broadcast_to(np.arange(hx.ntotal), prod.shape), -prod), axis=1)[:, :10]
    assert (r.ids == order).all()
    assert (r.dists.astype(np.int64) == np.take_along_axis(prod, order, 1)).all()
    # fewer candidates than K: padded with -1 / -inf
    tiny = ib.add_vectors(base[:5], hx.centroids, hx.codebook, metric="ip")
    r2 = oracle.search(oracle.OracleIndex(tiny), q[:2], 10, hx.nlist, 20)
    assert (r2.ids[:, 5:] == -1).all() and np.isneginf(r2.dists[:, 5:]).all()


def test_ip_seil_equals_naive_layout_with_soar_assignment():
    base, hx = _ip_index(24)
    assert (hx.assign[:, 0] != hx.assign[:, 1]).all() and hx.nrefs > 0
    ox = oracle.OracleIndex(hx)
    q = small_queries(7, 40, hx.d)
    for nprobe in (1, 3, 7, hx.nlist):
        a = oracle.search(ox, q, 10, nprobe, 60, layout="seil", trace=True)
        b = oracle.search(ox, q, 10, nprobe, 60, layout="naive")
        assert (a.cand_ids == b.cand_ids).all() and (a.cand_acc == b.cand_acc).all()
        assert (a.ids == b.ids).all() and (a.dists == b.dists).all()
        assert a.push_count.max() <= 1 and a.block_count.max() <= 1


# --- other block sizes (BLK_SZ of Alg. 4; Section 6.4) -------------------------------------------

@pytest.mark.parametrize("blk", [16, 64])
def test_other_block_sizes_same_results_and_dco_identity(blk):
    base = datagen.random_vectors(31, 4000, 16)
    g = np.random.Generator(np.random.PCG64(130))
    centers = g.uniform(-1, 1, size=(8, 16)).astype(np.float32)
    base = (centers[g.integers(0, 8, size=4000)] + 0.25 * base).astype(np.float32)
    ref = ib.build_index(base, 16, 8, seed=31, coarse_iters=8, pq_iters=8)
    hx = ib.add_vectors(base, ref.centroids, ref.codebook, blk=blk)
    assert (hx.assign == ref.assign).all() and hx.blk == blk
    q = small_queries(8, 30, 16)
    a = hx.assign.astype(np.int64)
    cells, cnt = np.unique(a[:, 0] * hx.nlist + a[:, 1], return_counts=True)
    c1, c2 = cells // hx.nlist, cells % hx.nlist
    members = np.bincount(a[:, 0], minlength=hx.nlist) + np.bincount(a[:, 1][a[:, 0] != a[:, 1]], minlength=hx.nlist)
    for nprobe in (1, 4, 9, hx.nlist):
        r = oracle.search(oracle.OracleIndex(hx), q, 10, nprobe, 50, trace=True)
        want = oracle.search(oracle.OracleIndex(ref), q, 10, nprobe, 50)
        naive = oracle.search(oracle.OracleIndex(hx), q, 10, nprobe, 50, layout="naive")
        # the block size changes the layout and the DCO, never the candidates or the results
        assert (r.cand_ids == want.cand_ids).all() and (r.ids == want.ids).all()
        assert (r.cand_ids == naive.cand_ids).all()
        assert r.push_count.max() <= 1 and r.block_count.max() <= 1
        for i in range(len(q)):
            probed = np.zeros(hx.nlist, dtype=bool)
            probed[r.probes[i]] = True
            both = probed[c1] & probed[c2] & (c1 != c2)
            assert r.dco[i] == members[probed].sum() - blk * (cnt[both] // blk).sum()


@pytest.mark.parametrize("blk", [16, 32, 64])
def test_ablation_dco_formula_equals_the_oracles_count(blk):
    # the block-size table of the ablation takes its DCO from Section 5.2's cost analysis; the
    # oracle counts the same number by scoring
    from paper_2601_07183_amd import ablation
    base = datagen.random_vectors(31, 4000, 16)
    ref = ib.build_index(base, 16, 8, seed=31, coarse_iters=4, pq_iters=4)
    hx = ib.add_vectors(base, ref.centroids, ref.codebook, blk=blk, strict=(blk != 64))
    q = datagen.random_vectors(32, 30, 16)
    for nprobe in (1, 5, 16):
        r = oracle.search(oracle.OracleIndex(hx), q, 10, nprobe, 50)
        assert (ablation.seil_dco(hx.assign, 16, r.probes, blk) == r.dco).all()
