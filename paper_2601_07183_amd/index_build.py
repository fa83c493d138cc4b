"""Deterministic host-side index construction (Alg. 1 of the paper: AddVectors).

Produces, from base vectors, everything the search path takes as input:
coarse centroids (k-means), PQ codebook and 4-bit codes (Section 2.2), the two list ids per
vector chosen by RairAssign (Alg. 3, AIR metric of Theorem 1), and the SEIL list layout written by
SeilInsert (Alg. 4) for a single batch.  The result is a `HostIndex` in a canonical host layout
that both the CPU oracle and the device upload consume; neither of them is imported here.

Construction is not on the measured path.  It is numpy plus torch used as a dense-algebra
library, seeded, and reproducible on a given machine.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

BLK = 32  # items per block (BLK_SZ in Alg. 4) unless a builder is told otherwise


@dataclass
class HostIndex:
    d: int
    M: int
    nlist: int
    ntotal: int
    centroids: np.ndarray          # [nlist][d] f32
    codebook: np.ndarray           # [M][16][d/M] f32
    # SEIL layout (Section 5.1): a flat array of 32-item blocks; list L owns
    # [shared_begin[L], +shared_cnt[L]) followed directly by [misc_begin[L], +misc_cnt[L]).
    codes: np.ndarray              # [nblocks][32][M/2] u8, low nibble = even subspace
    ids: np.ndarray                # [nblocks][32] i64, -1 = empty slot
    other: np.ndarray              # [nblocks][32] i32, other-list id for misc items, -1 elsewhere
    list_shared_begin: np.ndarray  # [nlist] i64
    list_shared_cnt: np.ndarray    # [nlist] i32
    list_misc_begin: np.ndarray    # [nlist] i64
    list_misc_cnt: np.ndarray      # [nlist] i32
    list_ref_begin: np.ndarray     # [nlist] i64
    list_ref_cnt: np.ndarray       # [nlist] i32
    ref_owner: np.ndarray          # [nrefs] i32
    ref_block_begin: np.ndarray    # [nrefs] i64
    ref_nblocks: np.ndarray        # [nrefs] i32
    raw: np.ndarray                # [ntotal][d] f32 or u8
    # per-vector view of the same index (the naive "every list holds its members" reading)
    assign: np.ndarray             # [ntotal][2] i32, assign[:,0] <= assign[:,1]
    vec_codes: np.ndarray          # [ntotal][M/2] u8
    params: dict = field(default_factory=dict)
    # "l2": squared Euclidean distance; "ip": inner product (larger is better), the metric of the
    # index that Section 6.4 applies SEIL to
    metric: str = "l2"

    @property
    def blk(self) -> int:
        """Items per block (BLK_SZ of Alg. 4); the device path is built for 32."""
        return int(self.ids.shape[1])

    @property
    def nblocks(self) -> int:
        return int(self.ids.shape[0])

    @property
    def nrefs(self) -> int:
        return int(self.ref_owner.shape[0])

    @property
    def raw_is_u8(self) -> bool:
        return self.raw.dtype == np.uint8


# ----------------------------------------------------------------------------------------------
# Dense helpers.  torch is used as a BLAS with threads (and the GPU when one is visible, which
# only makes construction faster; the search path never sees torch).
# ----------------------------------------------------------------------------------------------

def _device():
    return torch.device("cuda") if torch.cuda.is_available() else torch.device("cpu")


def _nearest(x: np.ndarray, c: np.ndarray, chunk: int = 131072):
    """Index of and squared distance to the nearest row of c for every row of x (GEMM form)."""
    dev = _device()
    ct = torch.from_numpy(np.ascontiguousarray(c, dtype=np.float32)).to(dev)
    cn = (ct.double() ** 2).sum(1).float()
    idx = np.empty(x.shape[0], dtype=np.int64)
    dist = np.empty(x.shape[0], dtype=np.float32)
    for lo in range(0, x.shape[0], chunk):
        xs = torch.from_numpy(np.ascontiguousarray(x[lo:lo + chunk], dtype=np.float32)).to(dev)
        g = cn[None, :] - 2.0 * (xs @ ct.T)
        dmin, i = g.min(1)
        idx[lo:lo + chunk] = i.cpu().numpy()
        dist[lo:lo + chunk] = (dmin + (xs * xs).sum(1)).cpu().numpy()
    return idx, dist


# ----------------------------------------------------------------------------------------------
# k-means (Lloyd).  Any deterministic choice is valid: the index is an input to the search path.
# ----------------------------------------------------------------------------------------------

def kmeans(x: np.ndarray, k: int, iters: int, seed: int, max_train: int | None = None) -> np.ndarray:
    g = np.random.Generator(np.random.PCG64(seed))
    n = x.shape[0]
    if max_train is not None and n > max_train:
        x = x[np.sort(g.choice(n, size=max_train, replace=False))]
        n = max_train
    x = np.ascontiguousarray(x, dtype=np.float32)
    c = x[np.sort(g.choice(n, size=k, replace=False))].copy()
    xt = torch.from_numpy(x).double()
    for _ in range(iters):
        idx, dist = _nearest(x, c)
        cnt = np.bincount(idx, minlength=k)
        s = torch.zeros((k, x.shape[1]), dtype=torch.float64)
        s.index_add_(0, torch.from_numpy(idx), xt)
        newc = c.astype(np.float64)
        nz = cnt > 0
        newc[nz] = s.numpy()[nz] / cnt[nz, None]
        # an empty cluster restarts on the point currently worst served
        empty = np.flatnonzero(cnt == 0)
        if empty.size:
            far = np.argsort(-dist, kind="stable")[:empty.size]
            newc[empty] = x[far]
        c = newc.astype(np.float32)
    return c


# ----------------------------------------------------------------------------------------------
# Product quantisation with 16 codewords per sub-quantizer (Section 2.2)
# ----------------------------------------------------------------------------------------------

def _sub_dist(xs: "torch.Tensor", cb: "torch.Tensor") -> "torch.Tensor":
    """xs [n][M][dsub], cb [M][16][dsub] -> squared distances [n][M][16], summed left to right."""
    dist = None
    for t in range(xs.shape[2]):
        diff = xs[:, :, None, t] - cb[None, :, :, t]
        dist = diff * diff if dist is None else dist + diff * diff
    return dist


def train_pq(x: np.ndarray, M: int, iters: int, seed: int, max_train: int = 32768) -> np.ndarray:
    g = np.random.Generator(np.random.PCG64(seed))
    n, d = x.shape
    dsub = d // M
    if n > max_train:
        x = x[np.sort(g.choice(n, size=max_train, replace=False))]
        n = max_train
    dev = _device()
    xs = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(dev).reshape(n, M, dsub)
    init = np.sort(g.choice(n, size=16, replace=False))
    cb = xs[torch.from_numpy(init).to(dev)].permute(1, 0, 2).double().contiguous()   # [M][16][dsub]
    # identical sub-vectors would give duplicate codewords; nudge them apart deterministically
    cb += torch.arange(16, dtype=torch.float64, device=dev)[None, :, None] * 1e-6
    xs64 = xs.double()
    moff = (torch.arange(M, device=dev) * 16)[None, :]
    for _ in range(iters):
        a = _sub_dist(xs, cb.float()).argmin(-1)                              # [n][M]
        key = (a + moff).reshape(-1)
        cnt = torch.bincount(key, minlength=16 * M).double()
        tot = torch.zeros((16 * M, dsub), dtype=torch.float64, device=dev)
        tot.index_add_(0, key, xs64.reshape(-1, dsub))
        nz = cnt > 0
        flat = cb.reshape(16 * M, dsub)
        flat[nz] = tot[nz] / cnt[nz, None]
    return cb.float().cpu().numpy()


def pq_encode(x: np.ndarray, cb: np.ndarray, chunk: int = 65536) -> np.ndarray:
    """PQEncoding: code[m] = nearest codeword of sub-vector m, first minimum on ties.
    Returns the packed form [n][M/2] with subspace 2i in the low nibble of byte i."""
    n, d = x.shape
    M, _, dsub = cb.shape
    dev = _device()
    out = np.empty((n, M // 2), dtype=np.uint8)
    cbt = torch.from_numpy(np.ascontiguousarray(cb, dtype=np.float32)).to(dev)
    chunk = max(1024, min(chunk, (1 << 27) // (M * 16)))
    for lo in range(0, n, chunk):
        xs = torch.from_numpy(np.ascontiguousarray(x[lo:lo + chunk], dtype=np.float32)).to(dev)
        dist = _sub_dist(xs.reshape(-1, M, dsub), cbt)
        # first minimum: argmin of (distance, codeword id)
        dmin = dist.min(-1, keepdim=True).values
        ids = torch.arange(16, device=dev)[None, None, :].expand_as(dist)
        code = torch.where(dist == dmin, ids, 16).min(-1).values.to(torch.uint8)
        out[lo:lo + chunk] = (code[:, 0::2] | (code[:, 1::2] << 4)).cpu().numpy()
    return out


# ----------------------------------------------------------------------------------------------
# RairAssign (Alg. 3)
# ----------------------------------------------------------------------------------------------

def air_loss(v: np.ndarray, cand_centroids: np.ndarray, lam: float) -> np.ndarray:
    """loss[i] = ||r_i||^2 + lam * <r_0, r_i>, r_i = centroid_i - v  (Alg. 3, the loop body).
    v: [n][d]; cand_centroids: [n][ncand][d] ordered by distance to v.  float64."""
    r = cand_centroids.astype(np.float64) - v.astype(np.float64)[:, None, :]
    return (r * r).sum(-1) + lam * (r * r[:, :1, :]).sum(-1)


def rair_assign(x: np.ndarray, centroids: np.ndarray, lam: float = 0.5, n_cands: int = 10,
                strict: bool = True, chunk: int = 32768) -> np.ndarray:
    """Two list ids per vector, returned ordered (smaller id first) as Alg. 3 does.
    With strict=False the secondary list may equal the primary one (the vector is then stored
    once, cell (i,i)); with strict=True candidate 0 is excluded from the argmin (SRAIR).
    FindNearestLists shortlists by a GEMM; the candidates are then re-scored directly in float64
    and ordered by (distance, list id)."""
    n = x.shape[0]
    nlist = centroids.shape[0]
    n_cands = min(n_cands, nlist)
    dev = _device()
    out = np.empty((n, 2), dtype=np.int32)
    c32 = torch.from_numpy(np.ascontiguousarray(centroids, dtype=np.float32)).to(dev)
    cn = (c32.double() ** 2).sum(1).float()
    c64 = c32.double()
    start = 1 if strict else 0
    for lo in range(0, n, chunk):
        xs = torch.from_numpy(np.ascontiguousarray(x[lo:lo + chunk], dtype=np.float32)).to(dev)
        g = cn[None, :] - 2.0 * (xs @ c32.T)
        cand = torch.topk(g, n_cands, dim=1, largest=False).indices
        cand = torch.sort(cand, dim=1).values
        r = c64[cand] - xs.double()[:, None, :]                # [chunk][ncand][d]
        dist = (r * r).sum(-1)
        key = torch.sort(dist, dim=1, stable=True).indices     # stable: ties keep the lower id
        cand = torch.gather(cand, 1, key)
        r = torch.gather(r, 1, key[:, :, None].expand_as(r))
        loss = (r * r).sum(-1) + lam * (r * r[:, :1, :]).sum(-1)
        first = cand[:, 0]
        if start >= n_cands:
            second = first
        else:
            # first minimum of the loss over candidates start..
            sub = loss[:, start:]
            lmin = sub.min(1, keepdim=True).values
            pos = torch.where(sub == lmin, torch.arange(sub.shape[1], device=dev)[None, :],
                              sub.shape[1]).min(1).values
            second = torch.gather(cand, 1, (pos + start)[:, None])[:, 0]
        out[lo:lo + chunk, 0] = torch.minimum(first, second).cpu().numpy()
        out[lo:lo + chunk, 1] = torch.maximum(first, second).cpu().numpy()
    return out


def soar_loss(v: np.ndarray, cand_centroids: np.ndarray, lam: float) -> np.ndarray:
    """SOAR's criterion as Section 2.3 and Table 1 state it: loss[i] = ||r_i||^2 +
    lam * (<r_0, r_i> / ||r_0||)^2 with r_i = v - centroid_i (the second term is 0 when r_0 = 0).
    v: [n][d]; cand_centroids: [n][ncand][d] ordered by distance to v.  float64."""
    r = v.astype(np.float64)[:, None, :] - cand_centroids.astype(np.float64)
    n0 = (r[:, 0, :] ** 2).sum(-1)
    proj2 = (r * r[:, :1, :]).sum(-1) ** 2 / np.where(n0 > 0, n0, 1.0)[:, None]
    return (r * r).sum(-1) + lam * np.where(n0[:, None] > 0, proj2, 0.0)


def soar_assign(x: np.ndarray, centroids: np.ndarray, lam: float = 1.0, n_cands: int = 10,
                chunk: int = 32768) -> np.ndarray:
    """Two list ids per vector by SOAR (Section 2.3): the nearest centroid, and among the other
    n_cands - 1 nearest the one of least ||r'||^2 + lam (r.r' / ||r||)^2, i.e. a second residual
    as orthogonal to the first as the distances allow.  Returned ordered, smaller id first."""
    n = x.shape[0]
    nlist = centroids.shape[0]
    n_cands = min(n_cands, nlist)
    out = np.empty((n, 2), dtype=np.int32)
    c64 = centroids.astype(np.float64)
    cn = (c64 ** 2).sum(1)
    for lo in range(0, n, chunk):
        xs = x[lo:lo + chunk].astype(np.float64)
        g = cn[None, :] - 2.0 * (xs @ c64.T)
        cand = np.argpartition(g, n_cands - 1, axis=1)[:, :n_cands] if n_cands < nlist else \
            np.tile(np.arange(nlist), (xs.shape[0], 1))
        cand = np.sort(cand, axis=1)
        dist = ((c64[cand] - xs[:, None, :]) ** 2).sum(-1)
        key = np.argsort(dist, axis=1, kind="stable")               # ties keep the lower id
        cand = np.take_along_axis(cand, key, axis=1)
        first = cand[:, 0]
        if n_cands < 2:
            second = first
        else:
            loss = soar_loss(xs, c64[cand], lam)[:, 1:]
            second = np.take_along_axis(cand[:, 1:], loss.argmin(1)[:, None], axis=1)[:, 0]
        out[lo:lo + chunk, 0] = np.minimum(first, second)
        out[lo:lo + chunk, 1] = np.maximum(first, second)
    return out


# ----------------------------------------------------------------------------------------------
# SeilInsert (Alg. 4), one batch
# ----------------------------------------------------------------------------------------------

def seil_insert(assign: np.ndarray, vec_codes: np.ndarray, vec_ids: np.ndarray, nlist: int,
                blk: int = BLK):
    """Lay the items out as Alg. 4 does for a single batch, with `blk` items per block (blk_SZ;
    32 by default, the size the device path is built for; Section 6.4 also looks at 16 and 64).

    Items are sorted by {listID1, listID2, vec_id}; a cell (i,j) of `nitems` items yields
    nitems // blk full blocks stored once, in list i's shared area, and nitems % blk leftovers that
    go to the miscellaneous area of list i and, when j != i, also of list j, each tagged with the
    other list id.  List j gets a reference entry (i, nblocks, first block) -- emitted only when
    nblocks >= 1.  Within a list, shared blocks precede miscellaneous blocks; only the last
    miscellaneous block of a list may be partly filled.
    """
    n = assign.shape[0]
    hb = vec_codes.shape[1]
    l1 = assign[:, 0].astype(np.int64)
    l2 = assign[:, 1].astype(np.int64)
    assert (l1 <= l2).all()
    order = np.lexsort((vec_ids, l2, l1))
    s1, s2 = l1[order], l2[order]
    cell_key = s1 * nlist + s2
    first = np.flatnonzero(np.concatenate([[True], cell_key[1:] != cell_key[:-1]])) if n else \
        np.zeros(0, dtype=np.int64)
    c_start = first
    c_n = np.diff(np.concatenate([first, [n]]))
    c_l1, c_l2 = s1[first], s2[first]
    c_nb = c_n // blk
    c_nm = c_n % blk
    ncell = first.size

    # pass 1: per-list block and leftover counts
    list_nb = np.bincount(c_l1, weights=c_nb, minlength=nlist).astype(np.int64)
    list_nm = np.bincount(c_l1, weights=c_nm, minlength=nlist).astype(np.int64)
    two = c_l1 != c_l2
    list_nm += np.bincount(c_l2[two], weights=c_nm[two], minlength=nlist).astype(np.int64)
    list_mb = (list_nm + blk - 1) // blk
    list_tot = list_nb + list_mb
    list_begin = np.concatenate([[0], np.cumsum(list_tot)[:-1]]).astype(np.int64)
    shared_begin = list_begin
    misc_begin = list_begin + list_nb
    nblocks = int(list_tot.sum())

    codes = np.zeros((nblocks * blk, hb), dtype=np.uint8)
    ids = np.full(nblocks * blk, -1, dtype=np.int64)
    other = np.full(nblocks * blk, -1, dtype=np.int32)

    # pass 2a: full blocks of each cell, contiguous, in list l1's shared area
    excl = np.cumsum(c_nb) - c_nb                      # blocks of earlier cells (global order)
    list_first_cell_excl = np.zeros(nlist, dtype=np.int64)
    # cells are sorted by l1, so the blocks of earlier cells of the same list are excl - (excl at
    # the list's first cell)
    firstcell_of_list = np.full(nlist, -1, dtype=np.int64)
    if ncell:
        fc = np.flatnonzero(np.concatenate([[True], c_l1[1:] != c_l1[:-1]]))
        firstcell_of_list[c_l1[fc]] = fc
        list_first_cell_excl[c_l1[fc]] = excl[fc]
    c_bbegin = shared_begin[c_l1] + (excl - list_first_cell_excl[c_l1])

    cell_of_item = np.repeat(np.arange(ncell), c_n)
    off = np.arange(n) - c_start[cell_of_item]
    in_shared = off < (c_nb[cell_of_item] * blk)
    src = order[in_shared]
    dst = c_bbegin[cell_of_item[in_shared]] * blk + off[in_shared]
    codes[dst] = vec_codes[src]
    ids[dst] = vec_ids[src]

    # pass 2b: leftovers, appended to list l1 and (if different) list l2 in cell order
    m_item = np.flatnonzero(~in_shared)                # positions in the sorted array
    m_cell = cell_of_item[m_item]
    a_dest = c_l1[m_cell]
    a_tag = c_l2[m_cell]
    sel2 = two[m_cell]
    b_dest = c_l2[m_cell][sel2]
    b_tag = c_l1[m_cell][sel2]
    e_dest = np.concatenate([a_dest, b_dest])
    e_tag = np.concatenate([a_tag, b_tag])
    e_pos = np.concatenate([m_item, m_item[sel2]])     # sorted position = (cell, offset) order
    eo = np.lexsort((e_pos, e_dest))
    e_dest, e_tag, e_pos = e_dest[eo], e_tag[eo], e_pos[eo]
    cnt = np.bincount(e_dest, minlength=nlist)
    assert (cnt == list_nm).all()
    rank = np.arange(e_dest.size) - np.repeat(np.cumsum(cnt) - cnt, cnt)
    dst = misc_begin[e_dest] * blk + rank
    src = order[e_pos]
    codes[dst] = vec_codes[src]
    ids[dst] = vec_ids[src]
    other[dst] = e_tag

    # reference entries: list l2 of every two-list cell that has at least one full block
    rsel = np.flatnonzero(two & (c_nb > 0))
    ro = np.lexsort((rsel, c_l2[rsel]))
    rsel = rsel[ro]
    ref_owner = c_l1[rsel].astype(np.int32)
    ref_block_begin = c_bbegin[rsel].astype(np.int64)
    ref_nblocks = c_nb[rsel].astype(np.int32)
    ref_cnt = np.bincount(c_l2[rsel], minlength=nlist).astype(np.int32)
    ref_begin = (np.cumsum(ref_cnt) - ref_cnt).astype(np.int64)

    return dict(
        codes=codes.reshape(nblocks, blk, hb), ids=ids.reshape(nblocks, blk),
        other=other.reshape(nblocks, blk),
        list_shared_begin=shared_begin.astype(np.int64), list_shared_cnt=list_nb.astype(np.int32),
        list_misc_begin=misc_begin.astype(np.int64), list_misc_cnt=list_mb.astype(np.int32),
        list_ref_begin=ref_begin, list_ref_cnt=ref_cnt,
        ref_owner=ref_owner, ref_block_begin=ref_block_begin, ref_nblocks=ref_nblocks,
    )


# ----------------------------------------------------------------------------------------------
# AddVectors (Alg. 1)
# ----------------------------------------------------------------------------------------------

def build_index(base: np.ndarray, nlist: int, M: int, *, lam: float = 0.5, n_cands: int = 10,
                strict: bool = True, seed: int = 0, coarse_iters: int = 20, pq_iters: int = 25,
                assign: np.ndarray | None = None, metric: str = "l2", blk: int = BLK) -> HostIndex:
    """Train centroids and codebook on `base`, then add all of `base` as one batch.
    `assign` overrides the assignment (tests use it for random and adversarial cell structures).
    metric "ip": the index is searched by inner product and its second lists come from SOAR
    (lam is then SOAR's weight) instead of RairAssign."""
    n, d = base.shape
    assert d % M == 0 and M % 2 == 0
    centroids = kmeans(base, nlist, coarse_iters, seed * 7 + 1, max_train=256 * nlist)
    codebook = train_pq(base, M, pq_iters, seed * 7 + 2)
    return add_vectors(base, centroids, codebook, lam=lam, n_cands=n_cands, strict=strict,
                       assign=assign, metric=metric, blk=blk)


def add_vectors(base: np.ndarray, centroids: np.ndarray, codebook: np.ndarray, *,
                lam: float = 0.5, n_cands: int = 10, strict: bool = True,
                assign: np.ndarray | None = None, metric: str = "l2", blk: int = BLK) -> HostIndex:
    n, d = base.shape
    nlist = centroids.shape[0]
    M = codebook.shape[0]
    assert metric in ("l2", "ip")
    if assign is None:
        assign = soar_assign(base, centroids, lam=lam, n_cands=n_cands) if metric == "ip" else \
            rair_assign(base, centroids, lam=lam, n_cands=n_cands, strict=strict)
    assign = np.ascontiguousarray(assign, dtype=np.int32)
    vec_codes = pq_encode(base, codebook)
    vec_ids = np.arange(n, dtype=np.int64)
    lay = seil_insert(assign, vec_codes, vec_ids, nlist, blk=blk)
    return HostIndex(
        d=d, M=M, nlist=nlist, ntotal=n,
        centroids=np.ascontiguousarray(centroids, dtype=np.float32),
        codebook=np.ascontiguousarray(codebook, dtype=np.float32),
        raw=np.ascontiguousarray(base), assign=assign, vec_codes=vec_codes,
        params=dict(lam=lam, n_cands=n_cands, strict=strict), metric=metric, **lay)


# ----------------------------------------------------------------------------------------------
# Later batches and deletion (Section 5.1's second-batch rules; the deletion rule of Section 6.1)
# ----------------------------------------------------------------------------------------------

def _block_owner(hx: HostIndex):
    """Per block: the list that stores it and whether it is a miscellaneous block (-1: unused)."""
    nb = hx.nblocks
    owner = np.full(nb, -1, dtype=np.int64)
    is_misc = np.zeros(nb, dtype=bool)
    for begin, cnt, misc in ((hx.list_shared_begin, hx.list_shared_cnt, False),
                             (hx.list_misc_begin, hx.list_misc_cnt, True)):
        cnt = cnt.astype(np.int64)
        lists = np.repeat(np.arange(hx.nlist), cnt)
        blk = np.repeat(begin.astype(np.int64) - (np.cumsum(cnt) - cnt), cnt) + np.arange(int(cnt.sum()))
        owner[blk] = lists
        is_misc[blk] = misc
    return owner, is_misc


def append_batch(hx: HostIndex, new: np.ndarray, *, lam: float = 0.5, n_cands: int = 10,
                 strict: bool = True, assign: np.ndarray | None = None) -> HostIndex:
    """Add a further batch of vectors to an index; their ids continue after the existing ones.

    The batch is grouped into cells on its own (Alg. 4).  The full blocks of its cells are appended
    to the shared blocks of the list that stores them and get a NEW reference entry in the other
    list, after that list's existing entries -- a list may then hold several entries to one owner.
    Its leftovers are appended to the miscellaneous items of their lists, so the partly filled
    last block of the earlier batches fills up before a new block starts.  Existing items keep
    their order.  The result is again one shared range and one miscellaneous range per list, the
    form the search side reads; block numbers change, ids do not.
    """
    n0, nlist = hx.ntotal, hx.nlist
    BLK = hx.blk
    new = np.ascontiguousarray(new, dtype=hx.raw.dtype)
    if assign is None:
        assign = rair_assign(new, hx.centroids, lam=lam, n_cands=n_cands, strict=strict)
    assign = np.ascontiguousarray(assign, dtype=np.int32)
    new_codes = pq_encode(new, hx.codebook)
    new_ids = np.arange(n0, n0 + new.shape[0], dtype=np.int64)
    lay = seil_insert(assign, new_codes, new_ids, nlist, blk=BLK)
    hb = hx.codes.shape[2]

    o_sb, o_sc = hx.list_shared_begin.astype(np.int64), hx.list_shared_cnt.astype(np.int64)
    b_sb, b_sc = lay["list_shared_begin"].astype(np.int64), lay["list_shared_cnt"].astype(np.int64)

    def misc_items(ids, other, codes, mb, mc):
        """Valid miscellaneous items in list order: (list, flat slot) of each."""
        mc = mc.astype(np.int64)
        lists = np.repeat(np.arange(nlist), mc)
        blk = np.repeat(mb.astype(np.int64) - (np.cumsum(mc) - mc), mc) + np.arange(int(mc.sum()))
        slots = (blk[:, None] * BLK + np.arange(BLK)[None, :]).reshape(-1)
        lists = np.repeat(lists, BLK)
        ok = ids.reshape(-1)[slots] >= 0
        return lists[ok], slots[ok]

    o_ml, o_ms = misc_items(hx.ids, hx.other, hx.codes, hx.list_misc_begin, hx.list_misc_cnt)
    b_ml, b_ms = misc_items(lay["ids"], lay["other"], lay["codes"], lay["list_misc_begin"],
                            lay["list_misc_cnt"])
    o_mn = np.bincount(o_ml, minlength=nlist).astype(np.int64)
    b_mn = np.bincount(b_ml, minlength=nlist).astype(np.int64)

    sc = o_sc + b_sc
    mc = (o_mn + b_mn + BLK - 1) // BLK
    tot = sc + mc
    begin = np.concatenate([[0], np.cumsum(tot)[:-1]]).astype(np.int64)
    sb, mb = begin, begin + sc
    nblocks = int(tot.sum())
    codes = np.zeros((nblocks * BLK, hb), dtype=np.uint8)
    ids = np.full(nblocks * BLK, -1, dtype=np.int64)
    other = np.full(nblocks * BLK, -1, dtype=np.int32)

    def copy_shared(src, src_sb, src_sc, dst_first):
        lists = np.repeat(np.arange(nlist), src_sc)
        k = np.arange(int(src_sc.sum())) - np.repeat(np.cumsum(src_sc) - src_sc, src_sc)
        s_blk = src_sb[lists] + k
        d_blk = dst_first[lists] + k
        s = (s_blk[:, None] * BLK + np.arange(BLK)[None, :]).reshape(-1)
        t = (d_blk[:, None] * BLK + np.arange(BLK)[None, :]).reshape(-1)
        codes[t] = src["codes"].reshape(-1, hb)[s]
        ids[t] = src["ids"].reshape(-1)[s]
        other[t] = src["other"].reshape(-1)[s]

    old = dict(codes=hx.codes, ids=hx.ids, other=hx.other)
    copy_shared(old, o_sb, o_sc, sb)
    copy_shared(lay, b_sb, b_sc, sb + o_sc)

    def copy_misc(src, lists, slots, first_rank):
        cnt = np.bincount(lists, minlength=nlist)
        rank = np.arange(lists.size) - np.repeat(np.cumsum(cnt) - cnt, cnt)
        t = mb[lists] * BLK + first_rank[lists] + rank
        codes[t] = src["codes"].reshape(-1, hb)[slots]
        ids[t] = src["ids"].reshape(-1)[slots]
        other[t] = src["other"].reshape(-1)[slots]

    copy_misc(old, o_ml, o_ms, np.zeros(nlist, dtype=np.int64))
    copy_misc(lay, b_ml, b_ms, o_mn)

    # reference entries: each list keeps its entries and gets the batch's after them
    o_rc, b_rc = hx.list_ref_cnt.astype(np.int64), lay["list_ref_cnt"].astype(np.int64)
    rc = o_rc + b_rc
    rb = (np.cumsum(rc) - rc).astype(np.int64)
    nrefs = int(rc.sum())
    ref_owner = np.zeros(nrefs, dtype=np.int32)
    ref_block_begin = np.zeros(nrefs, dtype=np.int64)
    ref_nblocks = np.zeros(nrefs, dtype=np.int32)

    def copy_refs(r_begin, r_cnt, owner, bbegin, nblk, src_sb, dst_first, first_rank):
        lists = np.repeat(np.arange(nlist), r_cnt)
        k = np.arange(int(r_cnt.sum())) - np.repeat(np.cumsum(r_cnt) - r_cnt, r_cnt)
        s = r_begin.astype(np.int64)[lists] + k
        t = rb[lists] + first_rank[lists] + k
        own = owner[s].astype(np.int64)
        ref_owner[t] = own
        ref_block_begin[t] = dst_first[own] + (bbegin[s].astype(np.int64) - src_sb[own])
        ref_nblocks[t] = nblk[s]

    copy_refs(hx.list_ref_begin, o_rc, hx.ref_owner, hx.ref_block_begin, hx.ref_nblocks, o_sb, sb,
              np.zeros(nlist, dtype=np.int64))
    copy_refs(lay["list_ref_begin"], b_rc, lay["ref_owner"], lay["ref_block_begin"],
              lay["ref_nblocks"], b_sb, sb + o_sc, o_rc)

    return HostIndex(
        d=hx.d, M=hx.M, nlist=nlist, ntotal=n0 + new.shape[0], centroids=hx.centroids,
        codebook=hx.codebook, codes=codes.reshape(nblocks, BLK, hb), ids=ids.reshape(nblocks, BLK),
        other=other.reshape(nblocks, BLK), list_shared_begin=sb, list_shared_cnt=sc.astype(np.int32),
        list_misc_begin=mb, list_misc_cnt=mc.astype(np.int32), list_ref_begin=rb,
        list_ref_cnt=rc.astype(np.int32), ref_owner=ref_owner, ref_block_begin=ref_block_begin,
        ref_nblocks=ref_nblocks, raw=np.concatenate([hx.raw, new]),
        assign=np.concatenate([hx.assign, assign]), vec_codes=np.concatenate([hx.vec_codes, new_codes]),
        params=dict(hx.params), metric=hx.metric)


def delete_ids(hx: HostIndex, ids_to_delete) -> HostIndex:
    """Remove vectors by id, in the order given, one position after the other.

    Every id has up to two positions (one per assigned list that stores it: a shared block is
    stored once).  A position in a shared block is invalidated in place (id -1; the block stays
    and is still scored, minus that slot).  A position in a miscellaneous block takes over the
    last miscellaneous item of the same list, which shrinks the area by one item; a last block
    that runs empty leaves the list's range (its storage is not reclaimed here).  Ids of other
    vectors, raw vectors and block numbers do not change; a deleted vector's row of `assign`
    becomes (-1, -1).
    """
    BLK = hx.blk
    codes = hx.codes.reshape(-1, hx.codes.shape[2]).copy()
    ids = hx.ids.reshape(-1).copy()
    other = hx.other.reshape(-1).copy()
    assign = hx.assign.copy()
    misc_cnt = hx.list_misc_cnt.copy()
    owner, is_misc = _block_owner(hx)
    # id -> its positions
    slots = np.flatnonzero(ids >= 0)
    order = np.argsort(ids[slots], kind="stable")
    slots = slots[order]
    start = np.searchsorted(ids[slots], np.arange(hx.ntotal + 1))
    pos = {}                                            # positions of items that were moved
    misc_n = np.zeros(hx.nlist, dtype=np.int64)         # items in each list's miscellaneous area
    m_l = owner[slots // BLK][is_misc[slots // BLK]]
    misc_n += np.bincount(m_l, minlength=hx.nlist)
    misc_begin = hx.list_misc_begin.astype(np.int64)
    for x in np.asarray(ids_to_delete, dtype=np.int64).reshape(-1):
        if x < 0 or x >= hx.ntotal or assign[x, 0] < 0:
            raise KeyError(f"id {int(x)} is not in the index")
        where = pos.pop(int(x), None)
        if where is None:
            where = [int(p) for p in slots[start[x]:start[x + 1]]]
        for p in where:
            assert ids[p] == x
            if not is_misc[p // BLK]:
                ids[p] = -1
                continue
            L = int(owner[p // BLK])
            last = int(misc_begin[L] * BLK + misc_n[L] - 1)
            if last != p:
                y = int(ids[last])
                codes[p], ids[p], other[p] = codes[last], y, other[last]
                wy = pos.get(y)
                if wy is None:
                    wy = [int(t) for t in slots[start[y]:start[y + 1]]]
                pos[y] = [p if t == last else t for t in wy]
            ids[last], other[last] = -1, -1
            codes[last] = 0
            misc_n[L] -= 1
            misc_cnt[L] = (misc_n[L] + BLK - 1) // BLK
        assign[x] = -1
    nb = hx.nblocks
    return HostIndex(
        d=hx.d, M=hx.M, nlist=hx.nlist, ntotal=hx.ntotal, centroids=hx.centroids,
        codebook=hx.codebook, codes=codes.reshape(nb, BLK, -1), ids=ids.reshape(nb, BLK),
        other=other.reshape(nb, BLK), list_shared_begin=hx.list_shared_begin,
        list_shared_cnt=hx.list_shared_cnt, list_misc_begin=hx.list_misc_begin,
        list_misc_cnt=misc_cnt.astype(np.int32), list_ref_begin=hx.list_ref_begin,
        list_ref_cnt=hx.list_ref_cnt, ref_owner=hx.ref_owner, ref_block_begin=hx.ref_block_begin,
        ref_nblocks=hx.ref_nblocks, raw=hx.raw, assign=assign, vec_codes=hx.vec_codes,
        params=dict(hx.params), metric=hx.metric)


def save_index(hx: HostIndex, path: str) -> None:
    """Write a host index to one .npz file (arrays as they are, scalars and parameters as JSON)."""
    import dataclasses
    import json
    arrays, meta = {}, {}
    for f in dataclasses.fields(hx):
        val = getattr(hx, f.name)
        if isinstance(val, np.ndarray):
            arrays[f.name] = val
        else:
            meta[f.name] = val
    meta["params"] = {k: (v.item() if isinstance(v, np.generic) else v) for k, v in dict(hx.params).items()}
    with open(path, "wb") as fh:
        np.savez(fh, _meta=np.frombuffer(json.dumps(meta, default=str).encode(), dtype=np.uint8), **arrays)


def load_index(path: str) -> HostIndex:
    """Read what save_index wrote (no pickled objects are loaded)."""
    import json
    with np.load(path, allow_pickle=False) as z:
        meta = json.loads(bytes(z["_meta"]).decode())
        arrays = {k: z[k] for k in z.files if k != "_meta"}
    return HostIndex(**arrays, **meta)
