"""Assignment-strategy ablation on a synthetic workload (Section 6.3 of the paper, off its datasets):
single assignment, naive redundant assignment (lambda = 0: the two nearest lists), SRAIR (strict)
and RAIR (not strict) at a given lambda, all on the same centroids and codebook and all through the
same GPU search path.  Prints recall@K, distance computations per query (DCO, deterministic) and a
quick rate per nprobe, as a markdown table.

    python -m paper_2601_07183_amd.ablation --workload sift1m
"""
import argparse
import time

import numpy as np


def main():
    import torch
    from . import binding, datagen, index_build as ib
    import bench                                          # ground truth and recall helpers

    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="sift1m")
    ap.add_argument("--base-size", type=int, default=0)
    ap.add_argument("--lam", type=float, default=0.5)
    ap.add_argument("--nprobes", default="4,8,16,32,64")
    args = ap.parse_args()
    binding.load()
    w = datagen.WORKLOADS[args.workload]
    if args.base_size:
        w = datagen.scaled(w, args.base_size)
    base, q = datagen.make_base(w), datagen.make_queries(w)
    gt = bench.ground_truth(base, q, w.k)
    centroids = ib.kmeans(base, w.nlist, 20, w.seed * 7 + 1, max_train=256 * w.nlist)
    codebook = ib.train_pq(base, w.M, 25, w.seed * 7 + 2)
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
