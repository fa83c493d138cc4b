"""Assignment-strategy ablation on a synthetic workload (Section 6.3 of the paper, off its datasets):
single assignment, naive redundant assignment (lambda = 0: the two nearest lists), SRAIR (strict)
and RAIR (not strict) at a given lambda, all on the same centroids and codebook and all through the
same GPU search path.  Prints recall@K, distance computations per query (DCO, deterministic) and a
quick rate per nprobe, as a markdown table.  With --sweep it varies lambda and N_CANDS instead
(Figure 14's axes) and prints, per setting, the share of vectors stored twice, the blocks SEIL
stores against two plain copies, and the cheapest nprobe that reaches the target recall with its
DCO next to the DCO of the same probes without SEIL (every member of every probed list scored,
Section 6.3's with/without comparison).  With --blocks it varies BLK_SZ over 16, 32 and 64 (Section
6.4's block-size axis) for the timed index's assignment: blocks stored, vectors in shared blocks
and the DCO at the probes that reach the target recall -- from the layout rule of Alg. 4 and the
cost analysis of Section 5.2 (DCO = n_vec_selected - n_vec_shared); results do not depend on the
block size, and the device path itself is built for 32 (whose DCO here is checked against the
kernels' own count).  With --ip the index is searched by inner product (Section 6.4 applies SEIL
to a SOAR index): single assignment against SOAR's second lists, the latter with its DCO next to
the DCO of the same probes without SEIL.

    python -m paper_2601_07183_amd.ablation --workload sift1m
    python -m paper_2601_07183_amd.ablation --workload sift1m --sweep
    python -m paper_2601_07183_amd.ablation --workload sift1m --blocks
    python -m paper_2601_07183_amd.ablation --workload sphere10m --base-size 1000000 --ip
"""
import argparse
import time

import numpy as np


def plain_blocks(assign: np.ndarray, nlist: int) -> int:
    """32-item blocks that two plain copies would take: every list stores all of its items itself."""
    a = np.asarray(assign)
    cnt = np.bincount(a[:, 0], minlength=nlist)
    two = a[:, 0] != a[:, 1]
    cnt = cnt + np.bincount(a[two, 1], minlength=nlist)
    return int(((cnt + 31) // 32).sum())


def cheapest_nprobe(ix, dq, gt, w, target, recall_at_k, top=256):
    """Smallest nprobe whose recall reaches target (recall grows with nprobe), by bisection."""
    def at(nprobe):
        ids, _ = ix.search(dq, w.k, nprobe, w.refine_k)
        return recall_at_k(ids.cpu().numpy(), gt), float(ix.dco(dq.shape[0]).mean())
    lo, hi = 0, 1
    while hi < top and at(hi)[0] < target:
        lo, hi = hi, hi * 2
    hi = min(hi, top)
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if at(mid)[0] >= target:
            hi = mid
        else:
            lo = mid
    return (hi,) + at(hi)


def sweep(args, w, base, q, gt, centroids, codebook):
    import torch
    from . import binding, index_build as ib
    import bench
    dq = torch.from_numpy(q).cuda()
    print("| lambda | N_CANDS | strict | vectors stored twice | SEIL blocks | two plain copies | saved | "
          "nprobe for recall %.2f | recall@%d | DCO per query | DCO without SEIL | DCO saved |" % (args.target, w.k))
    print("|---|---|---|---|---|---|---|---|---|---|---|---|")
    settings = [(lam, 10, True) for lam in (0.0, 0.25, 0.5, 0.75, 1.0)]
    settings += [(0.5, nc, True) for nc in (2, 5, 20)]
    settings += [(0.5, 10, False)]
    for lam, nc, strict in settings:
        hx = ib.add_vectors(base, centroids, codebook, lam=lam, n_cands=nc, strict=strict)
        twice = float((hx.assign[:, 0] != hx.assign[:, 1]).mean())
        plain = plain_blocks(hx.assign, w.nlist)
        ix = binding.Index(hx)
        nprobe, rec, dco = cheapest_nprobe(ix, dq, gt, w, args.target, bench.recall_at_k)
        # without SEIL every probed list scores all of its members
        a = hx.assign
        two = a[:, 0] != a[:, 1]
        members = np.bincount(a[:, 0], minlength=w.nlist) + np.bincount(a[two, 1], minlength=w.nlist)
        pid, _ = ix.coarse(dq, nprobe)
        dco_plain = float(members[pid.cpu().numpy()].sum(1).mean())
        print(f"| {lam} | {nc} | {strict} | {twice:.3f} | {hx.nblocks:,} | {plain:,} | "
              f"{1 - hx.nblocks / plain:.1%} | {nprobe} | {rec:.4f} | {dco:,.0f} | {dco_plain:,.0f} | "
              f"{1 - dco / dco_plain:.1%} |", flush=True)
        ix.free()


def seil_dco(assign: np.ndarray, nlist: int, probes: np.ndarray, blk: int) -> np.ndarray:
    """DCO of every query under SEIL with `blk` items per block, from Section 5.2's cost analysis:
    the members of the probed lists, minus the items of full blocks of cells whose two lists are
    both probed (those blocks are stored, and scored, once)."""
    a = np.asarray(assign, dtype=np.int64)
    two = a[:, 0] != a[:, 1]
    members = np.bincount(a[:, 0], minlength=nlist) + np.bincount(a[two, 1], minlength=nlist)
    cells, cnt = np.unique(a[two, 0] * nlist + a[two, 1], return_counts=True)
    keep = cnt >= blk
    c1, c2, shared = cells[keep] // nlist, cells[keep] % nlist, (cnt[keep] // blk) * blk
    out = np.empty(len(probes), dtype=np.int64)
    for lo in range(0, len(probes), 256):
        p = probes[lo:lo + 256]
        probed = np.zeros((len(p), nlist), dtype=bool)
        np.put_along_axis(probed, p, True, axis=1)
        out[lo:lo + 256] = members[p].sum(1) - ((probed[:, c1] & probed[:, c2]) * shared[None, :]).sum(1)
    return out


def blocks(args, w, base, q, gt, centroids, codebook):
    import torch
    from . import binding, index_build as ib
    import bench
    dq = torch.from_numpy(q).cuda()
    hx = ib.add_vectors(base, centroids, codebook, lam=args.lam, strict=True)
    ix = binding.Index(hx)
    nprobe, rec, dco32 = cheapest_nprobe(ix, dq, gt, w, args.target, bench.recall_at_k)
    pid, _ = ix.coarse(dq, nprobe)
    probes = pid.cpu().numpy()
    ix.search(dq, w.k, nprobe, w.refine_k)
    counted = ix.dco(len(q))
    ix.free()
    two = hx.assign[:, 0] != hx.assign[:, 1]
    members = np.bincount(hx.assign[:, 0], minlength=w.nlist) + np.bincount(hx.assign[two, 1], minlength=w.nlist)
    plain = float(members[probes].sum(1).mean())
    print(f"strict AIR, lambda {args.lam}; nprobe {nprobe} reaches recall@{w.k} {rec:.4f}; DCO without SEIL {plain:,.0f}")
    print("| BLK_SZ | blocks stored | item slots | two plain copies (slots) | vectors in shared blocks | "
          "DCO per query | DCO saved | equals the kernels' count |")
    print("|---|---|---|---|---|---|---|---|")
    vec_ids = np.arange(hx.ntotal, dtype=np.int64)
    for blk in (16, 32, 64):
        lay = ib.seil_insert(hx.assign, hx.vec_codes, vec_ids, w.nlist, blk=blk)
        nb = lay["ids"].shape[0]
        shared = float(lay["list_shared_cnt"].sum()) * blk / hx.ntotal
        plain_slots = int((((members + blk - 1) // blk) * blk).sum())
        dco = seil_dco(hx.assign, w.nlist, probes, blk)
        same = bool((dco == counted).all()) if blk == 32 else None
        print(f"| {blk} | {nb:,} | {nb * blk:,} | {plain_slots:,} | {shared:.3f} | {dco.mean():,.0f} | "
              f"{1 - dco.mean() / plain:.2%} | {'-' if same is None else same} |", flush=True)


def ip_ground_truth(base: np.ndarray, queries: np.ndarray, k: int) -> np.ndarray:
    """Ids of the k largest inner products per query (ties: smaller id): a GPU matmul (a tool)
    shortlists k + 54 per query, float64 products re-rank them."""
    import torch
    b = torch.from_numpy(np.ascontiguousarray(base, dtype=np.float32)).cuda()
    out = []
    step = max(1, min(500, (1 << 30) // max(1, len(base))))
    for lo in range(0, len(queries), step):
        q = torch.from_numpy(queries[lo:lo + step]).cuda()
        cand = torch.topk(b @ q.T, k + 54, dim=0, largest=True).indices.T.contiguous()
        exact = (b[cand].double() * q.double()[:, None, :]).sum(-1)
        cand_sorted, perm = torch.sort(cand, dim=1)
        exact = torch.gather(exact, 1, perm)
        order = torch.sort(-exact, dim=1, stable=True).indices[:, :k]
        out.append(torch.gather(cand_sorted, 1, order).cpu().numpy())
    return np.concatenate(out)


def inner_product(args, w, base, q, centroids, codebook):
    """Single assignment against SOAR (lambda as given) under the inner-product metric."""
    import torch
    from . import binding, index_build as ib
    import bench
    base = np.ascontiguousarray(base, dtype=np.float32)
    gt = ip_ground_truth(base, q, w.k)
    dq = torch.from_numpy(q).cuda()
    near = ib.rair_assign(base, centroids, lam=0.0, n_cands=1, strict=False)
    print("| assignment | vectors stored twice | blocks | nprobe | recall@%d | DCO per query | DCO without SEIL | "
          "DCO saved | queries/s |" % w.k)
    print("|---|---|---|---|---|---|---|---|---|")
    for name, kw in (("single", dict(assign=near)), (f"SOAR (lambda {args.lam}) + SEIL", dict(lam=args.lam))):
        hx = ib.add_vectors(base, centroids, codebook, metric="ip", **kw)
        a = hx.assign
        two = a[:, 0] != a[:, 1]
        members = np.bincount(a[:, 0], minlength=w.nlist) + np.bincount(a[two, 1], minlength=w.nlist)
        ix = binding.Index(hx)
        for nprobe in [int(x) for x in args.nprobes.split(",")]:
            ids, _ = ix.search(dq, w.k, nprobe, w.refine_k)
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(3):
                ix.search(dq, w.k, nprobe, w.refine_k)
            torch.cuda.synchronize()
            sec = (time.perf_counter() - t) / 3
            dco = float(ix.dco(len(q)).mean())
            pid, _ = ix.coarse(dq, nprobe)
            plain = float(members[pid.cpu().numpy()].sum(1).mean())
            print(f"| {name} | {float(two.mean()):.3f} | {hx.nblocks:,} | {nprobe} | "
                  f"{bench.recall_at_k(ids.cpu().numpy(), gt):.4f} | {dco:,.0f} | {plain:,.0f} | "
                  f"{1 - dco / plain:.2%} | {len(q) / sec:,.0f} |", flush=True)
        ix.free()


def main():
    import torch
    from . import binding, datagen, index_build as ib
    import bench                                          # ground truth and recall helpers

    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="sift1m")
    ap.add_argument("--base-size", type=int, default=0)
    ap.add_argument("--lam", type=float, default=0.5)
    ap.add_argument("--nprobes", default="4,8,16,32,64")
    ap.add_argument("--sweep", action="store_true", help="vary lambda and N_CANDS instead")
    ap.add_argument("--blocks", action="store_true", help="vary BLK_SZ over 16, 32, 64 instead")
    ap.add_argument("--ip", action="store_true", help="inner-product metric: single assignment against SOAR + SEIL")
    ap.add_argument("--target", type=float, default=0.9, help="recall the sweep searches to")
    args = ap.parse_args()
    binding.load()
    w = datagen.WORKLOADS[args.workload]
    if args.base_size:
        w = datagen.scaled(w, args.base_size)
    base, q = datagen.make_base(w), datagen.make_queries(w)
    centroids = ib.kmeans(base, w.nlist, 20, w.seed * 7 + 1, max_train=256 * w.nlist)
    codebook = ib.train_pq(base, w.M, 25, w.seed * 7 + 2)
    if args.ip:
        return inner_product(args, w, base, q, centroids, codebook)
    gt = bench.ground_truth(base, q, w.k)
    if args.sweep:
        return sweep(args, w, base, q, gt, centroids, codebook)
    if args.blocks:
        return blocks(args, w, base, q, gt, centroids, codebook)
    near = ib.rair_assign(base, centroids, lam=0.0, n_cands=1, strict=False)       # (nearest, nearest)
    variants = [("single", dict(assign=near)),
                ("naive RA (lambda 0)", dict(lam=0.0, strict=True)),
                (f"SRAIR (lambda {args.lam})", dict(lam=args.lam, strict=True)),
                (f"RAIR (lambda {args.lam})", dict(lam=args.lam, strict=False))]
    dq = torch.from_numpy(q).cuda()
    print("| assignment | code bytes | vectors stored twice | nprobe | recall@%d | DCO per query | queries/s |" % w.k)
    print("|---|---|---|---|---|---|---|")
    for name, kw in variants:
        hx = ib.add_vectors(base, centroids, codebook, **kw)
        twice = float((hx.assign[:, 0] != hx.assign[:, 1]).mean())
        ix = binding.Index(hx)
        code_bytes, _ = ix.bytes()
        for nprobe in [int(x) for x in args.nprobes.split(",")]:
            ids, _ = ix.search(dq, w.k, nprobe, w.refine_k)
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(3):
                ix.search(dq, w.k, nprobe, w.refine_k)
            torch.cuda.synchronize()
            sec = (time.perf_counter() - t) / 3
            rec = bench.recall_at_k(ids.cpu().numpy(), gt)
            print(f"| {name} | {code_bytes / 1e6:.1f} MB | {twice:.3f} | {nprobe} | {rec:.4f} | "
                  f"{ix.dco(len(q)).mean():,.0f} | {len(q) / sec:,.0f} |", flush=True)
        ix.free()


if __name__ == "__main__":
    main()
