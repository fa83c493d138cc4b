"""HIP path vs CPU oracle, element by element, through the C ABI.  Needs an MI355X."""
import numpy as np
import pytest

from oracle import oracle
from paper_2601_07183_amd import datagen, index_build as ib

from conftest import small_queries

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def binding():
    from paper_2601_07183_amd import binding as b
    b.load()
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    return b


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _assert_dists(got, want):
    # bar: 1e-5 relative (the two sides use the same summation order, so this is normally 0)
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    fin = np.isfinite(want)
    assert (np.isfinite(got) == fin).all()
    assert (np.abs(got[fin] - want[fin]) <= 1e-5 * np.abs(want[fin])).all()
    assert (got[~fin] == want[~fin]).all()


def _compare_all_stages(binding, hx, q, k, nprobe, refine_k):
    print(f"case: n={hx.ntotal} d={hx.d} M={hx.M} nlist={hx.nlist} nq={len(q)} k={k} "
          f"nprobe={nprobe} refine_k={refine_k}", flush=True)
    ox = oracle.OracleIndex(hx)
    want = oracle.search(ox, q, k, nprobe, refine_k)
    ix = binding.Index(hx)
    try:
        dq = _dev(q)
        # coarse quantizer: ids exactly; distances within 1e-4 absolute + 1e-5 relative
        pid, pdist = ix.coarse(dq, nprobe)
        torch.cuda.synchronize()
        assert (pid.cpu().numpy() == want.probes).all()
        for i in range(0, len(q), max(1, len(q) // 8)):
            _, od = oracle.coarse(ox, q[i], nprobe)
            assert (np.abs(pdist[i].cpu().numpy() - od) <= 1e-4 + 1e-5 * np.abs(od)).all()
        # lookup tables: bit exact
        lut, bias, scale = ix.lut(dq)
        torch.cuda.synchronize()
        assert (lut.cpu().numpy() == want.lut).all()
        for i in range(0, len(q), max(1, len(q) // 8)):
            _, _, ob, osc = oracle.lut(ox, q[i])
            assert bias[i].item() == np.float32(ob) and scale[i].item() == np.float32(osc)
        for exact in (False, True):                  # MFMA list-major path, then exact-only path
            ix.set_scan_mode(exact)
            # scan on the ORACLE's tables and probe lists: integer work, bit exact
            cand, score, dco = ix.scan(_dev(want.lut), _dev(want.probes), refine_k)
            torch.cuda.synchronize()
            assert (cand.cpu().numpy() == want.cand_ids).all(), f"exact={exact}"
            assert (score.cpu().numpy() == want.cand_acc).all(), f"exact={exact}"
            assert (dco.cpu().numpy() == want.dco).all(), f"exact={exact}"
            # whole path
            ids, dists = ix.search(dq, k, nprobe, refine_k)
            torch.cuda.synchronize()
            assert (ids.cpu().numpy() == want.ids).all(), f"exact={exact}"
            _assert_dists(dists.cpu().numpy(), want.dists)
            assert (ix.dco(len(q)) == want.dco).all()
        # refine on the ORACLE's candidates
        rid, rd = ix.refine(dq, _dev(want.cand_ids), k)
        torch.cuda.synchronize()
        assert (rid.cpu().numpy() == want.ids).all()
        _assert_dists(rd.cpu().numpy(), want.dists)
    finally:
        ix.free()
    return want


@pytest.mark.parametrize("nprobe", [1, 4, 16, 64])
def test_tiny_workload_all_stages(binding, tiny_workload, nprobe):
    w, base, q, hx = tiny_workload
    _compare_all_stages(binding, hx, q, w.k, nprobe, w.refine_k)


@pytest.mark.parametrize("which", ["strict", "nonstrict", "int"])
def test_small_indexes(binding, which, small_index, small_index_nonstrict, small_index_int):
    base, hx = {"strict": small_index, "nonstrict": small_index_nonstrict,
                "int": small_index_int}[which]
    q = small_queries(40, 37, hx.d, integer=(which == "int"))     # ragged query count
    for nprobe, refine_k, k in ((1, 50, 10), (5, 33, 33), (hx.nlist, 100, 1)):
        _compare_all_stages(binding, hx, q, k, nprobe, refine_k)


@pytest.mark.parametrize("d,M", [(128, 64), (96, 48), (32, 16)])
def test_table_shapes_of_the_mfma_scan(binding, d, M):
    # the three table shapes the matrix-core scan is built for, on integer-valued data so that
    # refine ties are real; nprobe = nlist with bigK = 1024 overflows the survivor buffers
    # (first list shorter than bigK => no bound) and exercises the exact redo
    g = np.random.Generator(np.random.PCG64(d))
    centers = g.integers(30, 220, size=(12, d))
    base = np.clip(centers[g.integers(0, 12, size=6000)] + g.normal(0, 25, size=(6000, d)), 0, 255)
    base = np.rint(base).astype(np.float32)
    q = np.rint(np.clip(centers[g.integers(0, 12, size=45)] + g.normal(0, 25, size=(45, d)), 0, 255))
    q = q.astype(np.float32)
    hx = ib.build_index(base, 20, M, seed=3, coarse_iters=5, pq_iters=5)
    for nprobe, refine_k, k in ((2, 100, 10), (7, 100, 10), (20, 1024, 10), (20, 40, 40)):
        _compare_all_stages(binding, hx, q, k, nprobe, refine_k)


def test_exact_knn_when_everything_is_probed(binding, small_index_int):
    base, hx = small_index_int
    q = small_queries(41, 16, hx.d, integer=True)
    ix = binding.Index(hx)
    try:
        ids, dists = ix.search(_dev(q), 10, hx.nlist, 1024)
        torch.cuda.synchronize()
    finally:
        ix.free()
    # bigK = 1024 < N here, so compare against the oracle rather than brute force ...
    want = oracle.search(oracle.OracleIndex(hx), q, 10, hx.nlist, 1024)
    assert (ids.cpu().numpy() == want.ids).all()
    # ... and the distances, being integers, against int64 arithmetic
    d2 = ((q[:, None, :].astype(np.int64) - base[ids.cpu().numpy()].astype(np.int64)) ** 2).sum(-1)
    assert (dists.cpu().numpy().astype(np.int64) == d2).all()


def test_adversarial_layouts(binding):
    x = datagen.random_vectors(31, 900, 8)
    q = datagen.random_vectors(32, 30, 8)
    cents = ib.kmeans(x, 8, 5, 1)
    cb = ib.train_pq(x, 4, 5, 2)
    g = np.random.Generator(np.random.PCG64(9))
    cases = [
        np.tile(np.array([[2, 5]], dtype=np.int32), (900, 1)),
        np.sort(g.integers(0, 8, size=(900, 2)), axis=1).astype(np.int32),
        np.sort(np.array([[i % 8, (i // 8) % 8] for i in range(900)]), axis=1)[:300].astype(np.int32),
        np.tile(np.array([[3, 3]], dtype=np.int32), (900, 1)),
        np.tile(np.array([[0, 7]], dtype=np.int32), (5, 1)),           # fewer items than k
    ]
    for asg in cases:
        hx = ib.add_vectors(x[:len(asg)], cents, cb, assign=asg)
        for nprobe in (1, 3, 8):
            _compare_all_stages(binding, hx, q, 5, nprobe, 40)


@pytest.mark.parametrize("d,M,strict", [(16, 8, True), (16, 8, False), (128, 64, True)])
def test_search_after_later_batches_and_deletion(binding, d, M, strict):
    # an index that grew in three batches, lost a quarter of its vectors (holes in shared blocks,
    # moved miscellaneous items, lists with several entries to one owner) and then grew again
    g = np.random.Generator(np.random.PCG64(d + M))
    centers = g.integers(30, 220, size=(10, d))
    pick = lambda n: np.rint(np.clip(centers[g.integers(0, 10, size=n)] + g.normal(0, 25, size=(n, d)),
                                     0, 255)).astype(np.float32)
    base, q = pick(6400), pick(45)
    hx = ib.build_index(base[:3000], 20, M, seed=5, coarse_iters=5, pq_iters=5, strict=strict)
    hx = ib.append_batch(hx, base[3000:4500], strict=strict)
    hx = ib.append_batch(hx, base[4500:6000], strict=strict)
    for nprobe, refine_k, k in ((3, 100, 10), (20, 60, 10)):
        _compare_all_stages(binding, hx, q, k, nprobe, refine_k)
    gone = g.choice(hx.ntotal, size=1500, replace=False)
    # and every item of the largest list's first shared blocks, which the bound's sample reads
    big = int(np.argmax(hx.list_shared_cnt))
    first = hx.ids[hx.list_shared_begin[big]:hx.list_shared_begin[big] + 2].reshape(-1)
    gone = np.unique(np.concatenate([gone, first[first >= 0]]))
    hx = ib.delete_ids(hx, gone)
    for nprobe, refine_k, k in ((1, 100, 10), (3, 100, 10), (7, 40, 40), (20, 1024, 10)):
        want = _compare_all_stages(binding, hx, q, k, nprobe, refine_k)
        assert not np.isin(want.ids, gone).any()
    hx = ib.append_batch(hx, base[6000:], strict=strict)
    for nprobe, refine_k, k in ((3, 100, 10), (20, 60, 10)):
        _compare_all_stages(binding, hx, q, k, nprobe, refine_k)


@pytest.mark.parametrize("d,M", [(128, 64), (96, 48), (32, 16)])
def test_bound_sample_on_the_matrix_cores(binding, d, M):
    # batches of 1,024 queries or more with at least four queries per list and bigK >= 64 take
    # their bound from a sample scored for queries grouped by first list: several tiles per list
    # (about 60 queries share a first list here), lists shorter than the sample, invalidated slots
    # in the sampled blocks, a sample with fewer than bigK items (bigK = 1024)
    g = np.random.Generator(np.random.PCG64(3 * d + M))
    centers = g.integers(30, 220, size=(12, d))
    pick = lambda n: np.rint(np.clip(centers[g.integers(0, 12, size=n)] + g.normal(0, 25, size=(n, d)),
                                     0, 255)).astype(np.float32)
    base, q = pick(9000), pick(1200)
    hx = ib.build_index(base, 20, M, seed=4, coarse_iters=5, pq_iters=5)
    for nprobe, refine_k, k in ((3, 100, 10), (20, 64, 10), (2, 1024, 10)):
        _compare_all_stages(binding, hx, q, k, nprobe, refine_k)
    big = int(np.argmax(hx.list_shared_cnt))
    first = hx.ids[hx.list_shared_begin[big]:hx.list_shared_begin[big] + 3].reshape(-1)
    gone = np.unique(np.concatenate([g.choice(hx.ntotal, size=2500, replace=False), first[first >= 0]]))
    hx = ib.delete_ids(hx, gone)
    for nprobe, refine_k, k in ((3, 100, 10), (7, 200, 20)):
        _compare_all_stages(binding, hx, q, k, nprobe, refine_k)


def test_bound_sample_on_the_matrix_cores_large_batch(binding):
    # more queries than the sample's grouping kernel keeps in registers per thread (12 x 1,024),
    # and more than 32 queries per first list on every list
    g = np.random.Generator(np.random.PCG64(77))
    d, M = 32, 16
    centers = g.integers(30, 220, size=(12, d))
    pick = lambda n: np.rint(np.clip(centers[g.integers(0, 12, size=n)] + g.normal(0, 25, size=(n, d)),
                                     0, 255)).astype(np.float32)
    base, q = pick(9000), pick(13500)
    hx = ib.build_index(base, 20, M, seed=6, coarse_iters=5, pq_iters=5)
    _compare_all_stages(binding, hx, q, 10, 4, 100)


@pytest.mark.parametrize("metric,d,M", [("l2", 32, 16), ("ip", 32, 16), ("l2", 128, 64), ("l2", 96, 48)])
def test_sample_ahead_of_the_probe_lists(binding, metric, d, M):
    # A batch large enough for the matrix-core sample over a directory large enough for the
    # matrix-core coarse quantizer: the sample is then taken from the list with the smallest key of
    # the score matrix while the probe lists are still being selected, and its ranking has to
    # find that list among them.  Half of the centroids are copies of the others moved by a few
    # units in the last place, so that for many queries the rounded keys and the exact distances
    # order the nearest lists differently; with nprobe 1 the sampled list is then not probed and
    # the query must get no bound rather than a wrong one.
    g = np.random.Generator(np.random.PCG64(31 + d))
    nlist = 64
    centers = g.uniform(-1, 1, size=(12, d)).astype(np.float32)
    pick = lambda n: (centers[g.integers(0, 12, size=n)] + 0.3 * g.standard_normal((n, d))).astype(np.float32)
    base, q = pick(20000), pick(1100)
    hx = ib.build_index(base, nlist, M, seed=2, coarse_iters=4, pq_iters=4, metric=metric)
    cents = hx.centroids.copy()
    cents[1::2] = cents[0::2] * np.float32(1 + 3e-7)
    hx2 = ib.add_vectors(base, cents, hx.codebook, metric=metric)
    for nprobe, refine_k in ((1, 64), (2, 100), (9, 100)):
        _compare_all_stages(binding, hx2, q, 10, nprobe, refine_k)


@pytest.mark.parametrize("count", [150, 600, 6000])
def test_identical_codes_tie_on_score(binding, count):
    # every vector identical: all scores tie, the order is decided by vector id alone, and every
    # scanned item survives any bound (with bigK = 64 the wave select takes up to 256 survivors,
    # the workgroup select up to 1,024, more overflow the buffer and go to the exact redo)
    x = np.tile(datagen.random_vectors(50, 1, 8), (count, 1))
    q = datagen.random_vectors(51, 9, 8)
    cents = datagen.random_vectors(52, 4, 8)
    cb = ib.train_pq(datagen.random_vectors(53, 300, 8), 4, 5, 2)
    g = np.random.Generator(np.random.PCG64(3))
    asg = np.sort(g.integers(0, 4, size=(count, 2)), axis=1).astype(np.int32)
    hx = ib.add_vectors(x, cents, cb, assign=asg)
    _compare_all_stages(binding, hx, q, 10, 4, 64)


def test_both_repairs_in_one_launch(binding):
    # two clumps of identical vectors in separate pairs of lists: a query next to the small clump
    # ends with 600 tied survivors (more than the wave select takes at bigK = 64: the
    # workgroup-wide select), a query next to the large one with 6,000 (its buffer overflows: the
    # exact redo).  Both lists of the repair launch are then non-empty in the same search.
    va = datagen.random_vectors(60, 1, 8)
    vb = va + np.float32(40)
    e = np.zeros((1, 8), np.float32)
    e[0, 0] = 0.5
    x = np.concatenate([np.tile(va, (600, 1)), np.tile(vb, (6000, 1))])
    cents = np.concatenate([va + e, va - e, vb + e, vb - e]).astype(np.float32)
    asg = np.array([[0, 1]] * 600 + [[2, 3]] * 6000, dtype=np.int32)
    cb = ib.train_pq(datagen.random_vectors(61, 300, 8), 4, 5, 2)
    noise = datagen.random_vectors(62, 9, 8) * np.float32(0.01)
    q = (np.concatenate([np.tile(va, (5, 1)), np.tile(vb, (4, 1))]) + noise).astype(np.float32)
    hx = ib.add_vectors(x, cents, cb, assign=asg)
    want = _compare_all_stages(binding, hx, q, 10, 2, 64)
    assert (want.probes[:5] < 2).all() and (want.probes[5:] >= 2).all()
    ix = binding.Index(hx)
    try:
        ix.search(_dev(q), 10, 2, 64)
        torch.cuda.synchronize()
        assert ix.scan_stats()["redone"] == 4            # the four queries next to the large clump
    finally:
        ix.free()


def test_survivor_log_runs_out_of_chunks(binding):
    # 120,000 identical vectors: every scanned item passes any bound, the survivor log of a small
    # batch runs out of chunks, every query is flagged and the exact kernel redoes them all
    count = 120_000
    x = np.tile(datagen.random_vectors(54, 1, 8), (count, 1))
    q = datagen.random_vectors(55, 30, 8)
    cents = datagen.random_vectors(56, 4, 8)
    cb = ib.train_pq(datagen.random_vectors(57, 300, 8), 4, 5, 2)
    g = np.random.Generator(np.random.PCG64(4))
    asg = np.sort(g.integers(0, 4, size=(count, 2)), axis=1).astype(np.int32)
    hx = ib.add_vectors(x, cents, cb, assign=asg)
    _compare_all_stages(binding, hx, q, 10, 4, 64)
    ix = binding.Index(hx)
    try:
        ix.search(_dev(q), 10, 4, 64)
        torch.cuda.synchronize()
        assert ix.scan_stats()["redone"] == len(q)       # the log did run out
    finally:
        ix.free()


def test_larger_dimensions_and_u8_raw(binding):
    # d = 192 (three 64-dimension folds), M = 96 (6 code dwords per lane), uint8 raw vectors
    g = np.random.Generator(np.random.PCG64(77))
    base = g.integers(0, 256, size=(4000, 192)).astype(np.uint8)
    q = g.integers(0, 256, size=(21, 192)).astype(np.float32)
    hx = ib.build_index(base.astype(np.float32), 24, 96, seed=5, coarse_iters=4, pq_iters=4)
    hx.raw = base
    _compare_all_stages(binding, hx, q, 10, 6, 100)


@pytest.mark.parametrize("nlist", [6100, 16384, 16500])
def test_many_short_lists(binding, nlist):
    # 6100 and 16,384 lists: the LDS grouping route with more than 48 KB of LDS per workgroup (128 KB
    # at its limit); 16,500 lists: queries are grouped by list with global counters, the separate
    # prefix kernel and the unit-table kernel.  The lists are short (one block each).
    base = datagen.random_vectors(91, 30000 if nlist < 10000 else 60000, 32)
    q = datagen.random_vectors(92, 70, 32)
    hx = ib.build_index(base, nlist, 16, seed=9, coarse_iters=2, pq_iters=4)
    _compare_all_stages(binding, hx, q, 10, 128, 60)


@pytest.mark.parametrize("d,nlist", [(32, 203), (64, 203), (96, 203), (128, 203), (256, 203),
                                     (32, 1100), (128, 2051), (200, 203), (528, 300)])
def test_coarse_shortlist_and_its_fallback(binding, d, nlist):
    # Lists at (nearly) the same distance: the matrix-core shortlist has to hand such queries to
    # the direct-form route, and ties are decided by list id on both sides.  From 1024 lists on,
    # the threshold comes from a sample of the row when that works, else from the radix select.
    g = np.random.Generator(np.random.PCG64(200 + d))
    nq = 77
    x = datagen.random_vectors(60 + d, 700, d)
    q = datagen.random_vectors(61 + d, nq, d)
    cb = ib.train_pq(x, d // 2 if d <= 256 else d // 8, 2, 2)
    asg = np.sort(g.integers(0, nlist, size=(len(x), 2)), axis=1).astype(np.int32)
    base_c = datagen.random_vectors(62 + d, nlist, d)
    dup = base_c.copy()
    dup[1::3] = dup[0::3][:len(dup[1::3])]                          # every third list repeats its neighbour
    near = (base_c[:1] + 1e-6 * g.standard_normal((nlist, d))).astype(np.float32)
    same = np.tile(base_c[:1], (nlist, 1))
    big = (base_c * 200.0 + 100.0).astype(np.float32)               # SIFT-like magnitudes
    for name, cents in (("random", base_c), ("dup", dup), ("near", near), ("same", same), ("big", big)):
        hx = ib.add_vectors(x, np.ascontiguousarray(cents), cb, assign=asg)
        ox = oracle.OracleIndex(hx)
        ix = binding.Index(hx)
        try:
            for nprobe in (1, 7, 64, nlist // 8, nlist):
                print(f"case: coarse d={d} nlist={nlist} centroids={name} nprobe={nprobe}", flush=True)
                qq = q * 200.0 + 100.0 if name == "big" else q
                pid, pdist = ix.coarse(_dev(qq.astype(np.float32)), nprobe)
                torch.cuda.synchronize()
                pid, pdist = pid.cpu().numpy(), pdist.cpu().numpy()
                for i in range(nq):
                    oi, od = oracle.coarse(ox, qq[i].astype(np.float32), nprobe)
                    assert (pid[i] == oi).all(), (name, nprobe, i)
                    assert (pdist[i] == od.astype(np.float32)).all()
        finally:
            ix.free()


def test_batch_permutation_and_split(binding, small_index):
    base, hx = small_index
    q = small_queries(42, 50, hx.d)
    ix = binding.Index(hx)
    try:
        ids, dists = ix.search(_dev(q), 10, 4, 40)
        perm = np.random.Generator(np.random.PCG64(1)).permutation(len(q))
        ids_p, dists_p = ix.search(_dev(q[perm]), 10, 4, 40)
        ids_s, _ = ix.search(_dev(q[:7]), 10, 4, 40)
        torch.cuda.synchronize()
        assert (ids_p.cpu().numpy() == ids.cpu().numpy()[perm]).all()
        assert (dists_p.cpu().numpy() == dists.cpu().numpy()[perm]).all()
        assert (ids_s.cpu().numpy() == ids.cpu().numpy()[:7]).all()
        # the same call twice gives the same bits
        ids2, dists2 = ix.search(_dev(q), 10, 4, 40)
        torch.cuda.synchronize()
        assert (ids2 == ids).all() and (dists2 == dists).all()
    finally:
        ix.free()


def test_batch_larger_than_one_internal_pass(binding):
    # rairs_search cuts a batch into passes of at most 65,536 queries that share one workspace and
    # the handle's two streams; 70,000 queries make two
    g = np.random.Generator(np.random.PCG64(78))
    d, M = 32, 16
    centers = g.integers(30, 220, size=(12, d))
    pick = lambda n: np.rint(np.clip(centers[g.integers(0, 12, size=n)] + g.normal(0, 25, size=(n, d)),
                                     0, 255)).astype(np.float32)
    base, q = pick(9000), pick(70000)
    hx = ib.build_index(base, 20, M, seed=7, coarse_iters=5, pq_iters=5)
    want = oracle.search(oracle.OracleIndex(hx), q, 10, 4, 100)
    ix = binding.Index(hx)
    try:
        for _ in range(2):                               # the second call reuses the grown workspace
            ids, dists = ix.search(_dev(q), 10, 4, 100)
            torch.cuda.synchronize()
            assert (ids.cpu().numpy() == want.ids).all()
            _assert_dists(dists.cpu().numpy(), want.dists)
            assert (ix.dco(len(q)) == want.dco).all()
    finally:
        ix.free()


@pytest.mark.parametrize("d,M,integer", [(16, 8, False), (128, 64, True), (96, 48, False), (32, 16, True)])
def test_inner_product_metric_with_soar_assignment(binding, d, M, integer):
    # Section 6.4's variant: an inner-product index whose second lists come from SOAR, in the same
    # SEIL layout and through the same kernels; probe ids, tables, candidates, ids and DCO bit-exact,
    # inner products within the distance bar (on integer data they are exact and ties are real)
    g = np.random.Generator(np.random.PCG64(5 * d + M))
    centers = g.uniform(-1, 1, size=(10, d)).astype(np.float32)
    pick = lambda n: (centers[g.integers(0, 10, size=n)] + 0.3 * g.standard_normal((n, d))).astype(np.float32)
    base, q = pick(5000), pick(53)
    if integer:
        base, q = (np.clip(np.rint(x * 60 + 128), 0, 255).astype(np.float32) for x in (base, q))
    hx = ib.build_index(base, 24, M, seed=8, coarse_iters=5, pq_iters=5, metric="ip", lam=1.0)
    assert hx.metric == "ip" and hx.nrefs > 0
    for nprobe, refine_k, k in ((1, 60, 10), (5, 100, 10), (24, 200, 20)):
        want = _compare_all_stages(binding, hx, q, k, nprobe, refine_k)
        assert (np.diff(want.dists, axis=1) <= 0).all()              # largest product first
    if integer:
        prod = q.astype(np.int64) @ base.astype(np.int64).T
        assert (want.dists.astype(np.int64) == np.take_along_axis(prod, want.ids, 1)).all()
    # nearly coincident and duplicated centroids: the shortlist's fallback under this metric
    cents = hx.centroids.copy()
    cents[1::3] = cents[0::3][:len(cents[1::3])]
    hx2 = ib.add_vectors(base, cents, hx.codebook, metric="ip", assign=hx.assign)
    _compare_all_stages(binding, hx2, q, 10, 7, 100)
    # RairAssign is a Euclidean criterion
    ix = binding.Index(hx)
    try:
        with pytest.raises(binding.RairsError) as e:
            ix.assign(_dev(base[:10]), 10, 0.5, True)
        assert e.value.code == -4
    finally:
        ix.free()


@pytest.mark.parametrize("d,M,metric", [(16, 16, "l2"), (24, 8, "l2"), (64, 16, "ip"), (80, 10, "l2"),
                                        (768, 192, "l2"), (96, 24, "ip")])
def test_lookup_tables_for_every_sub_vector_size(binding, d, M, metric):
    # the table kernel keeps the codewords in registers for sub-vectors of 1, 2 and 4 dimensions
    # and re-reads them otherwise (3 and 8 here); M = 192 gives a thread three groups of codes;
    # more queries than one workgroup takes, and a count that is not a multiple of it
    base = datagen.random_vectors(600 + d, 1500, d)
    q = datagen.random_vectors(601 + d, 21, d)
    hx = ib.build_index(base, 8, M, seed=5, coarse_iters=2, pq_iters=3, metric=metric)
    ox = oracle.OracleIndex(hx)
    ix = binding.Index(hx)
    try:
        lut, bias, scale = ix.lut(_dev(q))
        torch.cuda.synchronize()
        for i in range(len(q)):
            _, ol, ob, osc = oracle.lut(ox, q[i])
            assert (lut[i].cpu().numpy().reshape(-1) == np.asarray(ol).reshape(-1)).all(), i
            assert bias[i].item() == np.float32(ob) and scale[i].item() == np.float32(osc), i
    finally:
        ix.free()


@pytest.mark.parametrize("d,integer,metric", [(128, True, "l2"), (96, False, "l2"), (200, False, "ip"),
                                              (64, True, "ip")])
def test_refine_one_wave_per_query(binding, d, integer, metric):
    # Batches of 4,096 queries and more take the refine kernel that gives every query one wave
    # (smaller ones a workgroup): candidate lists with missing (-1) and out-of-range ids, fewer
    # candidates than K, duplicated base vectors (equal distances, ordered by id), byte and fp32
    # rows, a dimension with a partial round of 64, both metrics; K below and above the size up to
    # which the results are found by rank.  Expected: oracle distances of a sample of the queries,
    # ordered by (distance, id).
    g = np.random.Generator(np.random.PCG64(900 + d))
    n, nq = 2500, 4096 + 37
    base = datagen.random_vectors(40 + d, n, d)
    q = datagen.random_vectors(41 + d, nq, d)
    if integer:
        base, q = (np.clip(np.rint(x * 40 + 128), 0, 255).astype(np.float32) for x in (base, q))
    base[1::5] = base[0::5][:len(base[1::5])]                  # every fifth row twice
    hx = ib.build_index(base, 16, d // 2 if d // 2 <= 64 else 8, seed=3, coarse_iters=2, pq_iters=2, metric=metric)
    dist = oracle.ip if metric == "ip" else oracle.l2sqr
    ix = binding.Index(hx)
    try:
        for refine_k, k in ((100, 10), (100, 1), (128, 16), (40, 17), (10, 10), (100, 100)):
            print(f"case: refine d={d} integer={integer} metric={metric} refine_k={refine_k} k={k}", flush=True)
            cand = g.integers(0, n, size=(nq, refine_k)).astype(np.int64)
            for i in range(nq):                                 # distinct ids per query
                cand[i] = g.choice(n, size=refine_k, replace=False)
            cand[g.random(cand.shape) < 0.05] = -1
            cand[5::11, refine_k // 2:] = -1                    # short lists, some shorter than K
            cand[3::97, 0] = n + 5                              # not an id of the index
            rid, rd = ix.refine(_dev(q), _dev(cand), k)
            torch.cuda.synchronize()
            rid, rd = rid.cpu().numpy(), rd.cpu().numpy()
            for i in list(range(0, nq, 131)) + [5, 16, 3, 100, nq - 1]:
                ok = [c for c in cand[i] if 0 <= c < n]
                sc = np.array([np.float32(dist(q[i], base[c])) for c in ok], dtype=np.float32)
                key = -sc if metric == "ip" else sc
                order = sorted(range(len(ok)), key=lambda t: (key[t], ok[t]))[:k]
                want_ids = np.full(k, -1, dtype=np.int64)
                want_d = np.full(k, -np.inf if metric == "ip" else np.inf, dtype=np.float32)
                want_ids[:len(order)] = [ok[t] for t in order]
                want_d[:len(order)] = [sc[t] for t in order]
                assert (rid[i] == want_ids).all(), (i, rid[i], want_ids)
                _assert_dists(rd[i], want_d)
    finally:
        ix.free()


def test_inner_product_coarse_routes(binding):
    # 1,100 lists and d = 128: the matrix-core shortlist with its sampled threshold; d = 5: the
    # full direct-form route; negative and positive products
    for d, nlist in ((128, 1100), (5, 70), (64, 203)):
        g = np.random.Generator(np.random.PCG64(300 + d))
        x = datagen.random_vectors(70 + d, 600, d)
        q = datagen.random_vectors(71 + d, 41, d)
        cents = datagen.random_vectors(72 + d, nlist, d)
        Mq = 2 if d == 5 else d // 2
        if d == 5:
            x, q, cents = (np.pad(a, ((0, 0), (0, 1))) for a in (x, q, cents))     # 6 dimensions, M = 2
        cb = ib.train_pq(x, Mq, 2, 2)
        asg = np.sort(g.integers(0, nlist, size=(len(x), 2)), axis=1).astype(np.int32)
        hx = ib.add_vectors(x, np.ascontiguousarray(cents), cb, assign=asg, metric="ip")
        ox = oracle.OracleIndex(hx)
        ix = binding.Index(hx)
        try:
            for nprobe in (1, 9, nlist // 8, nlist):
                print(f"case: ip coarse d={hx.d} nlist={nlist} nprobe={nprobe}", flush=True)
                pid, pdot = ix.coarse(_dev(q), nprobe)
                torch.cuda.synchronize()
                for i in range(len(q)):
                    oi, od = oracle.coarse(ox, q[i], nprobe)
                    assert (pid[i].cpu().numpy() == oi).all()
                    assert (pdot[i].cpu().numpy() == od.astype(np.float32)).all()
        finally:
            ix.free()


@pytest.mark.parametrize("nq", [1, 7])
def test_search_graph_replays(binding, tiny_workload, nq):
    # a captured search replayed several times on new queries, with eager searches and
    # synchronisations of the same handle in between: every replay must equal the eager result
    w, base, q, hx = tiny_workload
    want = oracle.search(oracle.OracleIndex(hx), q, w.k, 16, w.refine_k)
    ix = binding.Index(hx)
    try:
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            dq = torch.zeros((nq, hx.d), dtype=torch.float32, device="cuda")
            ids = torch.full((nq, w.k), -7, dtype=torch.int64, device="cuda")
            dists = torch.zeros((nq, w.k), dtype=torch.float32, device="cuda")
            dq.copy_(_dev(q[:nq]))
            stream.synchronize()
            g = ix.graph(dq, w.k, 16, w.refine_k, ids, dists, stream)
            for rep in range(5):
                lo = (rep * nq) % (len(q) - nq)
                dq.copy_(_dev(q[lo:lo + nq]))
                ids.fill_(-7)
                g.launch(stream)
                stream.synchronize()
                assert (ids.cpu().numpy() == want.ids[lo:lo + nq]).all(), rep
                _assert_dists(dists.cpu().numpy(), want.dists[lo:lo + nq])
                # eager work of the same handle between replays (its own workspace)
                e_ids, _ = ix.search(_dev(q[:50]), w.k, 4 + rep, w.refine_k, stream=stream)
                stream.synchronize()
                assert e_ids.shape == (50, w.k)
            g.free()
            g.free()                                         # second free is a no-op
        with pytest.raises(binding.RairsError):
            ix.graph(dq, w.k, 16, w.refine_k, ids, dists, torch.cuda.default_stream())
    finally:
        ix.free()


def test_caller_owned_workspace(binding, tiny_workload):
    # rairs_workspace_bytes / rairs_set_workspace through the C ABI: a torch tensor serves as the
    # workspace; one byte too few is RAIRS_EWORKSPACE and enqueues nothing; the library's own
    # workspace and the caller's give the same bits
    import ctypes as C
    w, base, q, hx = tiny_workload
    lib = binding.load()
    want = oracle.search(oracle.OracleIndex(hx), q, w.k, 16, w.refine_k)
    ix = binding.Index(hx)
    try:
        dq = _dev(q)
        need = ix.workspace_bytes(len(q), 16, w.refine_k)
        assert need > 0 and ix.workspace_bytes(0, 16, w.refine_k) == 0
        assert ix.workspace_bytes(len(q) // 2, 8, w.refine_k) <= need       # monotone in its arguments
        with pytest.raises(binding.RairsError):
            ix.workspace_bytes(len(q), hx.nlist + 1, w.refine_k)
        ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
        ids = torch.full((len(q), w.k), -7, dtype=torch.int64, device="cuda")
        dists = torch.zeros((len(q), w.k), dtype=torch.float32, device="cuda")
        h, stream = ix._h, C.c_void_p(torch.cuda.current_stream().cuda_stream)
        args = (h, C.c_void_p(dq.data_ptr()), C.c_int64(len(q)), C.c_int(w.k), C.c_int(16), C.c_int(w.refine_k),
                C.c_void_p(ids.data_ptr()), C.c_void_p(dists.data_ptr()), stream)
        # too small by one byte: refused, outputs untouched
        assert lib.rairs_set_workspace(h, C.c_void_p(ws.data_ptr()), C.c_size_t(need - 1)) == 0
        assert lib.rairs_search(*args) == -5
        torch.cuda.synchronize()
        assert (ids == -7).all()
        # misaligned: refused
        assert lib.rairs_set_workspace(h, C.c_void_p(ws.data_ptr() + 8), C.c_size_t(need)) == -1
        # exactly enough
        assert lib.rairs_set_workspace(h, C.c_void_p(ws.data_ptr()), C.c_size_t(need)) == 0
        assert lib.rairs_search(*args) == 0
        torch.cuda.synchronize()
        assert (ids.cpu().numpy() == want.ids).all()
        _assert_dists(dists.cpu().numpy(), want.dists)
        assert (ix.dco(len(q)) == want.dco).all()
        # back to the handle's own workspace: same bits
        ix.use_own_workspace()
        ids2, dists2 = ix.search(dq, w.k, 16, w.refine_k)
        torch.cuda.synchronize()
        assert (ids2 == ids).all() and (dists2 == dists).all()
    finally:
        ix.free()


def test_argument_errors_and_empty_batch(binding, small_index):
    base, hx = small_index
    q = _dev(small_queries(43, 4, hx.d))
    ix = binding.Index(hx)
    try:
        empty = torch.empty((0, hx.d), dtype=torch.float32, device="cuda")
        ids, dists = ix.search(empty, 10, 4, 40)
        assert ids.shape == (0, 10)
        for kw in (dict(k=0, nprobe=4, refine_k=40), dict(k=50, nprobe=4, refine_k=40),
                   dict(k=10, nprobe=0, refine_k=40), dict(k=10, nprobe=hx.nlist + 1, refine_k=40)):
            with pytest.raises(binding.RairsError) as e:
                ix.search(q, **kw)
            assert e.value.code == -1
        with pytest.raises(binding.RairsError) as e:
            ix.search(q, 10, 4, binding.MAX_REFINE_K + 1)
        assert e.value.code == -4
    finally:
        ix.free()
    ix.free()                                               # second free is a no-op


def test_stage_timers(binding, tiny_workload):
    # the stage timers are measurement helpers: levels, the ring of recorded searches, errors
    w, base, q, hx = tiny_workload
    ix = binding.Index(hx)
    try:
        dq = _dev(q)
        with pytest.raises(binding.RairsError):
            ix.stage_ms()                                    # nothing recorded yet
        with pytest.raises(binding.RairsError):
            ix.set_profiling(7)
        ix.set_profiling(binding.PROFILE_SCAN_KERNEL)
        ix.search(dq, w.k, 16, w.refine_k)
        ms = ix.stage_ms()
        assert ms["scan_kernel"] > 0 and all(ms[k] == -1 for k in ms if k != "scan_kernel")
        ix.set_profiling(binding.PROFILE_STAGES)
        for _ in range(3):
            ids, _ = ix.search(dq, w.k, 16, w.refine_k)
        one, mean = ix.stage_ms(), ix.stage_ms_mean(3)
        assert all(v > 0 for v in one.values()) and all(v > 0 for v in mean.values())
        assert one["scan_kernel"] <= one["scan"]
        with pytest.raises(binding.RairsError):
            ix.stage_ms_mean(4)                              # only three recorded at this level
        ix.set_profiling(False)
        ids2, _ = ix.search(dq, w.k, 16, w.refine_k)
        torch.cuda.synchronize()
        assert (ids.cpu().numpy() == ids2.cpu().numpy()).all()
        with pytest.raises(binding.RairsError):
            ix.stage_ms()
    finally:
        ix.free()


@pytest.mark.parametrize("d,M", [(32, 16), (128, 64), (96, 48), (960, 240), (64, 64), (60, 6), (24, 2)])
def test_pq_encode_matches_the_oracle(binding, d, M):
    # sub-vectors of 2, 2, 2, 4, 1 (codebook in registers), 10 and 12 (codebook in LDS) dimensions;
    # ragged vector counts around the grid's stride; bit exact
    g = np.random.Generator(np.random.PCG64(d * 1000 + M))
    cb = g.standard_normal((M, 16, d // M)).astype(np.float32)
    cb[:, 11] = cb[:, 2]                                  # a tie in every sub-quantizer
    for n in (0, 1, 777, 20011):
        print(f"case: pq_encode d={d} M={M} n={n}", flush=True)
        x = g.standard_normal((n, d)).astype(np.float32)
        x[: n // 3] = np.round(x[: n // 3])              # integer-valued rows: more exact ties
        if n > 5:
            x[5] = cb[np.arange(M), (np.arange(M) * 7) % 16].reshape(-1)   # a vector made of codewords
        got = binding.pq_encode(_dev(cb), _dev(x) if n else torch.empty((0, d), device="cuda"))
        torch.cuda.synchronize()
        want = oracle.pq_encode(cb, x) if n else np.empty((0, M // 2), dtype=np.uint8)
        assert got.shape == want.shape and (got.cpu().numpy() == want).all()
    with pytest.raises(binding.RairsError):
        binding.pq_encode(_dev(np.zeros((3, 16, 2), dtype=np.float32)), _dev(np.zeros((4, 6), dtype=np.float32)))


def test_rair_assign_matches_the_oracle(binding, small_index, small_index_int, tiny_workload):
    # Alg. 3 on the GPU: candidates from the coarse kernels (full route for 16 lists, matrix-core
    # shortlist for 64), float64 loss; bit exact, also on integer data with its exact distance ties
    for which, (base, hx) in (("float", small_index), ("int", small_index_int),
                              ("tiny", (tiny_workload[1], tiny_workload[3]))):
        ix = binding.Index(hx)
        try:
            g = np.random.Generator(np.random.PCG64(23))
            x = np.concatenate([base[:700], small_queries(41, 333, hx.d, integer=(which == "int"))])
            x[3] = hx.centroids[5]                           # a vector that is a centroid: r_0 = 0
            for n_cands, lam, strict in ((10, 0.5, True), (10, 0.5, False), (1, 0.5, True), (7, 0.0, True),
                                         (32, 2.0, True), (hx.nlist + 5 if hx.nlist < 28 else 32, 0.25, False)):
                print(f"case: assign {which} n_cands={n_cands} lambda={lam} strict={strict}", flush=True)
                got = ix.assign(_dev(x), n_cands, lam, strict)
                torch.cuda.synchronize()
                want = oracle.rair_assign(hx.centroids, x, n_cands, lam, strict)
                assert (got.cpu().numpy() == want).all()
            assert ix.assign(torch.empty((0, hx.d), device="cuda"), 10, 0.5, True).shape == (0, 2)
            with pytest.raises(binding.RairsError):
                ix.assign(_dev(x), 0, 0.5, True)
            if hx.nlist > 32:
                with pytest.raises(binding.RairsError):
                    ix.assign(_dev(x), 33, 0.5, True)
        finally:
            ix.free()

