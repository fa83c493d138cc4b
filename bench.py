#!/usr/bin/env python3
"""Benchmark of the RAIRS query path on one MI355X.

One "step" = one rairs_search call over the whole query batch of the workload (coarse quantizer,
lookup tables, SEIL scan + top-bigK, refine), with queries, index and outputs resident in HBM.
The headline is queries per second at the smallest swept nprobe whose recall@10 (against exact
brute-force neighbours) is at least 0.9.  Prints ONE JSON line on stdout; everything else goes
to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# MI355X matrix peaks for int8: dense 5.0 POP/s; the 2:4-sparse instruction v_smfmac_i32_32x32x64_i8
# retires twice the K extent of the dense v_mfma_i32_32x32x32_i8 per pass (131,072 ops in 32 cycles
# per SIMD x 1,024 SIMDs x 2.4 GHz), i.e. twice that for the ops it stands for.
MFMA_I8_DENSE_POPS = 5.0
MFMA_I8_SPARSE_POPS = 10.1
LANE_OPS_PEAK = 256 * 64 * 2.4e9          # one 64-lane vector operation per compute unit and cycle

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "scan_kernel_hbm_traffic.md")


def measured_traffic(workload: str, nprobe: int, kernel: str):
    """HBM bytes per launch of the scan kernel from the tracked rocprofv3 counter summary
    (profiles/scan_kernel_hbm_traffic.md: FETCH_SIZE and WRITE_SIZE per dispatch, each scaled by
    what the same counter reads for a plain copy of known size), or None when the table has no
    row for this (workload, nprobe, kernel)."""
    try:
        rows = open(TRAFFIC_TABLE).read().splitlines()
    except OSError:
        return None
    for line in rows:
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 7 and cells[0] == workload and cells[1] == str(nprobe) and cells[2] == kernel:
            try:
                fetch_kib, fetch_f, write_kib, write_f = (float(cells[i].replace(",", "")) for i in (3, 4, 5, 6))
            except ValueError:
                continue
            return (fetch_kib * fetch_f + write_kib * write_f) * 1024.0
    return None


def physical_cores():
    """Cores (not SMT threads) that lscpu reports for the host, or None."""
    import subprocess
    try:
        out = subprocess.run(["lscpu"], capture_output=True, text=True, timeout=10).stdout
        per, sockets = None, None
        for line in out.splitlines():
            if line.startswith("Core(s) per socket:"):
                per = int(line.split(":")[1])
            elif line.startswith("Socket(s):"):
                sockets = int(line.split(":")[1])
        return per * sockets if per and sockets else None
    except Exception:
        return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def ground_truth(base: np.ndarray, queries: np.ndarray, k: int):
    """Exact kNN ids by brute force, ties by smaller id.  A GPU matmul (used as a tool) shortlists
    k + 54 candidates per query; they are re-ranked by direct float64 distances, and a few
    queries are re-checked against a full float64 scan."""
    import torch
    b = torch.empty((len(base), base.shape[1]), dtype=torch.float32, device="cuda")
    for lo in range(0, len(base), 1 << 22):               # uint8 bases are converted piecewise
        b[lo:lo + (1 << 22)] = torch.from_numpy(base[lo:lo + (1 << 22)]).cuda().float()
    bn = (b * b).sum(1)
    short = k + 54
    out = []
    step = max(1, min(500, (1 << 30) // max(1, len(base))))     # keep every tensor below 2^31 elements
    for lo in range(0, len(queries), step):
        q = torch.from_numpy(queries[lo:lo + step]).cuda()
        # (b @ q.T) rather than (q @ b.T): the latter returned garbage here for 10M-row b
        d2 = bn[:, None] - 2.0 * (b @ q.T)                                   # [n][nq]
        cand = torch.topk(d2, short, dim=0, largest=False).indices.T.contiguous()   # [nq][short]
        diff = b[cand].double() - q.double()[:, None, :]
        exact = (diff * diff).sum(-1)
        cand_sorted, perm = torch.sort(cand, dim=1)                         # ties: smaller id first
        exact = torch.gather(exact, 1, perm)
        order = torch.sort(exact, dim=1, stable=True).indices[:, :k]
        out.append(torch.gather(cand_sorted, 1, order).cpu().numpy())
    gt = np.concatenate(out)
    for i in range(0, len(queries), max(1, len(queries) // 5)):
        d2 = (b.double() - torch.from_numpy(queries[i]).cuda().double()[None, :]).pow(2).sum(1) \
            if len(base) <= (1 << 24) else None
        if d2 is None:                                        # very large base: check in pieces
            parts = [(b[lo:lo + (1 << 24)].double() - torch.from_numpy(queries[i]).cuda().double()[None, :])
                     .pow(2).sum(1) for lo in range(0, len(base), 1 << 24)]
            d2 = torch.cat(parts)
        kth = torch.sort(d2).values[k - 1].item()
        assert (d2[torch.from_numpy(gt[i]).cuda()] <= kth * (1 + 1e-9)).all().item(), \
            "ground truth check failed"
    del b, bn
    torch.cuda.empty_cache()
    return gt


def recall_at_k(ids: np.ndarray, gt: np.ndarray) -> float:
    hits = 0
    for a, b in zip(ids, gt):
        hits += len(set(a.tolist()) & set(b.tolist()))
    return hits / gt.size


def bench_pq_encode(args):
    """PQEncoding of the workload's base vectors with a codebook trained on them: vectors/s, the
    algorithmic HBM rate (vectors read once, codes written once) and the oracle's rate."""
    import torch
    from oracle import oracle
    from paper_2601_07183_amd import binding, datagen, index_build
    binding.load()
    w = datagen.WORKLOADS[args.workload]
    if args.base_size:
        w = datagen.scaled(w, args.base_size)
    base = datagen.make_base(w).astype(np.float32, copy=False)
    cb = index_build.train_pq(base, w.M, 8, w.seed * 7 + 2)
    dx, dcb = torch.from_numpy(base).cuda(), torch.from_numpy(cb).cuda()
    n, d = base.shape
    for _ in range(max(1, args.warmup)):
        codes = binding.pq_encode(dcb, dx)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(args.steps):
        codes = binding.pq_encode(dcb, dx)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.steps
    ns = min(n, 200_000)
    t = time.perf_counter()
    want = oracle.pq_encode(cb, base[:ns])
    cpu_s = time.perf_counter() - t
    same = bool((codes[:ns].cpu().numpy() == want).all())
    bytes_per_launch = float(n) * d * 4 + float(n) * (w.M // 2)
    gbs = bytes_per_launch / (ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "PQ encode rate", "value": round(n / (ms * 1e-3), 1), "unit": "vectors/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: N={n} d={d} M={w.M}x4bit", "codes_identical_to_oracle_on_sample": same},
        "roofline": {"kernel": "pq_encode_kernel", "bound": "hbm", "achieved": round(gbs, 1), "peak": 8000.0,
                     "unit": "GB/s", "frac": round(gbs / 8000.0, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": bytes_per_launch},
        # what bounds it: per (vector, sub-quantizer, codeword) dsub subtractions, dsub products,
        # dsub - 1 additions and three compare/select operations, none of them fused or packed,
        # against one 64-lane operation per compute unit and cycle (256 CUs, 2.4 GHz)
        "roofline_alu": {"kernel": "pq_encode_kernel", "bound": "alu",
                         "achieved": round(n / (ms * 1e-3) * w.M * 16 * (3 * (d // w.M) + 2) / 1e12, 2),
                         "peak": round(256 * 64 * 2.4e9 / 1e12, 2), "unit": "T lane-ops/s",
                         "frac": round(n / (ms * 1e-3) * w.M * 16 * (3 * (d // w.M) + 2) / (256 * 64 * 2.4e9), 4)},
        "cpu_baseline": {"value": round(ns / cpu_s, 1), "unit": "vectors/s", "cores": oracle.num_threads(),
                         "kind": "oracle", "sample": f"first {ns} vectors"}}))


def bench_assign(args):
    """RairAssign of the workload's base vectors against the index's centroids: vectors/s and the
    oracle's rate; the lists chosen are compared with the oracle's on a sample."""
    import torch
    from oracle import oracle
    from paper_2601_07183_amd import binding, datagen, index_build
    binding.load()
    w = datagen.WORKLOADS[args.workload]
    if args.base_size:
        w = datagen.scaled(w, args.base_size)
    base = datagen.make_base(w).astype(np.float32, copy=False)
    # a small index supplies the handle: its centroids are trained on the whole base
    hx = index_build.build_index(base[: min(len(base), 200_000)], w.nlist, w.M, seed=w.seed, coarse_iters=4,
                                 pq_iters=2)
    hx.centroids = index_build.kmeans(base, w.nlist, 20, w.seed * 7 + 1, max_train=256 * w.nlist)
    ix = binding.Index(hx)
    dx = torch.from_numpy(base).cuda()
    n, d = base.shape
    for _ in range(max(1, args.warmup)):
        pairs = ix.assign(dx, 10, 0.5, True)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(args.steps):
        pairs = ix.assign(dx, 10, 0.5, True)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.steps
    ns = min(n, 20_000)
    t = time.perf_counter()
    want = oracle.rair_assign(hx.centroids, base[:ns], 10, 0.5, True)
    cpu_s = time.perf_counter() - t
    same = bool((pairs[:ns].cpu().numpy() == want).all())
    print(json.dumps({
        "metric": "RairAssign rate", "value": round(n / (ms * 1e-3), 1), "unit": "vectors/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "dtype": "f32 coarse, f64 loss", "data": "synthetic",
        "config": {"workload": f"{w.name}: N={n} d={d} nlist={w.nlist} n_cands=10 lambda=0.5 strict",
                   "pairs_identical_to_oracle_on_sample": same},
        "cpu_baseline": {"value": round(ns / cpu_s, 1), "unit": "vectors/s", "cores": oracle.num_threads(),
                         "kind": "oracle", "sample": f"first {ns} vectors"}}))


def bench_incremental(args):
    """Search over an index that grew and shrank (the set-up of the paper's insertion/deletion
    experiment, Section 6.2: 800,000 vectors, then five batches of 40,000 insertions, then five
    batches of 40,000 deletions), timed and checked after each phase.  The mutations themselves
    run in the host builder; what is measured is the GPU search path on the resulting layouts."""
    import torch
    from paper_2601_07183_amd import binding, datagen, index_build as ib
    from oracle import oracle
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.load()
    w = datagen.WORKLOADS[args.workload]
    if args.base_size:
        w = datagen.scaled(w, args.base_size)
    nprobe = args.nprobe or 23
    base, queries = datagen.make_base(w), datagen.make_queries(w)
    n0, nb = int(w.n * 0.8), int(w.n * 0.04)
    dq = torch.from_numpy(queries).cuda()
    nq = len(queries)
    phases = []

    def measure(name, hx, live, host_sec, host_items):
        keep = np.flatnonzero(live)
        gt = keep[ground_truth(base[keep], queries, w.k)]
        ix = binding.Index(hx)
        ids, _ = ix.search(dq, w.k, nprobe, w.refine_k)
        for _ in range(args.warmup):
            ix.search(dq, w.k, nprobe, w.refine_k)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(args.steps):
            ix.search(dq, w.k, nprobe, w.refine_k)
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t) / args.steps
        got = ids.cpu().numpy()
        ncpu = args.cpu_queries or 100
        want = oracle.search(oracle.OracleIndex(hx), queries[:ncpu], w.k, nprobe, w.refine_k)
        code_bytes, _ = ix.bytes()
        point = {"phase": name, "vectors": int(live.sum()), "nblocks": hx.nblocks, "nrefs": hx.nrefs,
                 "code_bytes": code_bytes, "recall_at_10": round(recall_at_k(got, gt), 4),
                 "qps": round(nq / sec, 1), "ms_per_step": round(sec * 1e3, 4),
                 "dco_per_query": float(ix.dco(nq).mean()),
                 "ids_identical_to_oracle_on_sample": bool((got[:ncpu] == want.ids).all()),
                 "host_builder_items_per_s": None if not host_items else round(host_items / host_sec, 1)}
        ix.free()
        log(f"[bench] {point}")
        phases.append(point)

    t = time.perf_counter()
    hx = ib.build_index(base[:n0], w.nlist, w.M, seed=w.seed)
    live = np.zeros(w.n, dtype=bool)
    live[:n0] = True
    measure("built", hx, live[:hx.ntotal], time.perf_counter() - t, 0)
    t = time.perf_counter()
    for b in range(5):
        hx = ib.append_batch(hx, base[n0 + b * nb:n0 + (b + 1) * nb])
    live[:hx.ntotal] = True
    measure("after 5 insertion batches", hx, live[:hx.ntotal], time.perf_counter() - t, 5 * nb)
    one = ib.add_vectors(base[:hx.ntotal], hx.centroids, hx.codebook)
    measure("same vectors in one batch", one, live[:hx.ntotal], 1.0, 0)
    g = np.random.Generator(np.random.PCG64(w.seed + 5))
    gone = g.choice(hx.ntotal, size=5 * nb, replace=False)
    t = time.perf_counter()
    for b in range(5):
        hx = ib.delete_ids(hx, gone[b * nb:(b + 1) * nb])
    live[gone] = False
    measure("after 5 deletion batches", hx, live[:hx.ntotal], time.perf_counter() - t, 5 * nb)
    print(json.dumps({"metric": f"QPS over a grown and thinned index ({w.name}, 1 GPU, nprobe {nprobe})",
                      "value": phases[-1]["qps"], "unit": "queries/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup,
                      "ms_per_step": phases[-1]["ms_per_step"], "higher_is_better": True,
                      "dtype": "i8", "data": "synthetic",
                      "config": {"workload": f"{w.name}: {n0} vectors, then 5 x {nb} inserted, then "
                                             f"5 x {nb} deleted; nq={nq} k={w.k} refine_k={w.refine_k}",
                                 "nprobe": nprobe},
                      "phases": phases}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="sift1m")
    ap.add_argument("--nprobe", type=int, default=0, help="skip the sweep and time this nprobe")
    ap.add_argument("--target-recall", type=float, default=0.9)
    ap.add_argument("--cpu-queries", type=int, default=0, help="oracle sample size (0 = auto)")
    ap.add_argument("--sweep-out", default="")
    ap.add_argument("--base-size", type=int, default=0,
                    help="use the workload's generator and parameters at this smaller base size "
                         "(for profiling; the headline numbers are quoted at full size)")
    ap.add_argument("--recall-queries", type=int, default=0,
                    help="measure recall on the first N queries only (0 = all); for very large bases")
    ap.add_argument("--parity-queries", type=int, default=0,
                    help="at every swept nprobe, also compare the first N queries' ids and DCO with the "
                         "CPU oracle's (the protocol for the largest workload: N >= 1000)")
    ap.add_argument("--k", type=int, default=0, help="override K of the workload (second workloads: K = 1, 100)")
    ap.add_argument("--refine-k", type=int, default=0, help="override bigK = K * K_FACTOR")
    ap.add_argument("--nq", type=int, default=0, help="queries per step (default: the workload's batch)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the same search captured once as a HIP graph and replayed "
                         "(the mode for one query at a time: --nq 1)")
    ap.add_argument("--index-cache", default="",
                    help="directory to keep the built index and the ground truth in, and to read "
                         "them from when they are there (repeated profiling runs on one machine)")
    ap.add_argument("--copy-calibration", type=int, default=0,
                    help="only run a device-to-device copy of this many bytes three times (to "
                         "calibrate rocprofv3's FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--pq-encode", action="store_true",
                    help="measure rairs_pq_encode (a step of index construction) on the workload's base "
                         "vectors instead of the search path; prints a JSON line of its own")
    ap.add_argument("--assign", action="store_true",
                    help="measure rairs_assign (RairAssign, a step of index construction) on the "
                         "workload's base vectors; prints a JSON line of its own")
    ap.add_argument("--incremental", action="store_true",
                    help="search over an index that grew by five insertion batches and then lost five "
                         "deletion batches (Section 6.2's set-up); prints a JSON line of its own")
    args = ap.parse_args()
    if args.incremental:
        return bench_incremental(args)
    if args.pq_encode:
        return bench_pq_encode(args)
    if args.assign:
        return bench_assign(args)
    if args.copy_calibration:
        import torch
        n = args.copy_calibration // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        # the same copy, timed: what a plain streaming kernel reaches on this device (read + write)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        gbs = 10 * 2 * n * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        print(json.dumps({"copy_bytes_read": n * 4, "copy_bytes_written": n * 4, "repeats": 3,
                          "timed_repeats": 10, "copy_read_plus_write_GBs": round(gbs, 1)}))
        return
    if args.gpus != 1:
        log("bench.py measures one GPU; this build has no multi-GPU path: queries are independent, so more GPUs would each take a share of the batch. "
            "Run with --gpus 1.")
        sys.exit(2)

    import torch
    from paper_2601_07183_amd import binding, datagen, index_build
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.load()

    w = datagen.WORKLOADS[args.workload]
    if args.base_size:
        w = datagen.scaled(w, args.base_size)
    if args.k or args.refine_k or args.nq:
        from dataclasses import replace
        w = replace(w, k=args.k or w.k, refine_k=args.refine_k or w.refine_k, nq=args.nq or w.nq)
    t0 = time.time()
    base = datagen.make_base(w)
    queries = datagen.make_queries(w)
    log(f"[bench] workload {w.name}: base {base.shape} {base.dtype}, queries {queries.shape} "
        f"({time.time() - t0:.1f}s)")
    t0 = time.time()
    nrec = min(len(queries), args.recall_queries) if args.recall_queries else len(queries)
    cache = None
    if args.index_cache:
        os.makedirs(args.index_cache, exist_ok=True)
        cache = os.path.join(args.index_cache, f"{w.name}_{len(base)}_{w.nlist}_{w.M}_{w.k}_{nrec}")
    if cache and os.path.exists(cache + ".index.npz") and os.path.exists(cache + ".gt.npy"):
        hx = index_build.load_index(cache + ".index.npz")
        gt = np.load(cache + ".gt.npy")
        log(f"[bench] index and ground truth read from {cache}.* in {time.time() - t0:.1f}s")
    else:
        hx = index_build.build_index(base, w.nlist, w.M, seed=w.seed)
        log(f"[bench] index built in {time.time() - t0:.1f}s")
        t0 = time.time()
        gt = ground_truth(base, queries[:nrec], w.k)
        log(f"[bench] ground truth for {nrec} queries in {time.time() - t0:.1f}s")
        if cache:
            index_build.save_index(hx, cache + ".index.npz")
            np.save(cache + ".gt.npy", gt)
    shared_frac = float(hx.list_shared_cnt.sum()) * 32 / hx.ntotal
    log(f"[bench] index: nblocks={hx.nblocks} nrefs={hx.nrefs} vectors in shared blocks={shared_frac:.3f}")

    ix = binding.Index(hx)
    code_bytes, total_bytes = ix.bytes()
    dq = torch.from_numpy(queries).cuda()
    nq = len(queries)
    out_ids = torch.empty((nq, w.k), dtype=torch.int64, device="cuda")
    out_d = torch.empty((nq, w.k), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def run(nprobe, steps, profile=False):
        """steps calls back to back; returns (seconds, mean stage ms, mean bytes scanned)."""
        ix.set_profiling(profile)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):                          # no host wait between the steps
            ix.search(dq, w.k, nprobe, w.refine_k, out_ids, out_d, stream)
        torch.cuda.synchronize()
        sec = time.perf_counter() - t
        # every search recorded its own events; the library keeps the last 64 of them
        stage = ix.stage_ms_mean(min(steps, 64)) if profile and steps else {}
        return sec, stage

    # --- nprobe sweep: recall and a quick rate per point ---------------------------------
    parity_ox = None

    def measure_point(nprobe):
        nonlocal parity_ox
        run(nprobe, 1)
        got = out_ids.cpu().numpy()
        rec = recall_at_k(got[:nrec], gt)
        parity = None
        if args.parity_queries:
            from oracle import oracle
            if parity_ox is None:
                parity_ox = oracle.OracleIndex(hx)
            npar = min(args.parity_queries, nq)
            t = time.perf_counter()
            want = oracle.search(parity_ox, queries[:npar], w.k, nprobe, w.refine_k)
            parity = dict(queries=npar, ids_identical=bool((got[:npar] == want.ids).all()),
                          dco_identical=bool((ix.dco(nq)[:npar] == want.dco).all()),
                          oracle_seconds=round(time.perf_counter() - t, 1))
        sec, stage = run(nprobe, 3, profile=True)
        dco = ix.dco(nq)
        st = ix.scan_stats()
        point = dict(nprobe=nprobe, recall_at_10=round(rec, 4), qps=round(3 * nq / sec, 1), parity=parity,
                     ms_per_batch=round(sec / 3 * 1e3, 3), dco_per_query=float(dco.mean()),
                     stage_ms={k: round(v, 4) for k, v in stage.items()},
                     survivors_per_query=round(st["survivors"] / max(1, st["queries"]), 1),
                     queries_redone_exactly=st["redone"],
                     scan_stage_algorithmic_GBs=round(float(dco.sum()) * (w.M // 2) / (stage["scan"] * 1e-3) / 1e9, 1),
                     scan_kernel_algorithmic_GBs=round(float(dco.sum()) * (w.M // 2) / (stage["scan_kernel"] * 1e-3) / 1e9, 1))
        log("[bench] " + json.dumps(point))
        return point

    sweep = []
    chosen = args.nprobe or None
    below = None                                         # largest swept nprobe that misses the target
    for nprobe in ((args.nprobe,) if args.nprobe else w.nprobes):
        point = measure_point(nprobe)
        sweep.append(point)
        if point["recall_at_10"] >= args.target_recall:
            if chosen is None:
                chosen = nprobe
        elif chosen is None:
            below = nprobe
    if chosen is None:
        chosen = sweep[-1]["nprobe"]
        log(f"[bench] WARNING: recall {args.target_recall} not reached; timing nprobe={chosen}")
    elif not args.nprobe and below is not None:
        # the metric is the rate AT the target recall: the smallest nprobe that reaches it, found
        # by bisection between the sweep's last miss and first hit (recall grows with nprobe)
        lo, hi = below, chosen
        while hi - lo > 1:
            mid = (lo + hi) // 2
            point = measure_point(mid)
            sweep.append(point)
            if point["recall_at_10"] >= args.target_recall:
                hi = mid
            else:
                lo = mid
        chosen = hi
        sweep.sort(key=lambda p: p["nprobe"])
    rec_chosen = [p for p in sweep if p["nprobe"] == chosen][0]["recall_at_10"]
    qps_interp = None
    for a, b in zip(sweep, sweep[1:]):
        if a["recall_at_10"] < args.target_recall <= b["recall_at_10"]:
            f = (args.target_recall - a["recall_at_10"]) / (b["recall_at_10"] - a["recall_at_10"])
            qps_interp = a["qps"] + f * (b["qps"] - a["qps"])

    # --- the timed region: W warm-up steps, then exactly K steps ---------------------------
    # Only the dominant kernel is bracketed by events here (its mean duration is the roofline's
    # denominator); every further event between two kernels costs the step some microseconds.
    run(chosen, args.warmup, profile=binding.PROFILE_SCAN_KERNEL)
    sec, stage = run(chosen, args.steps, profile=binding.PROFILE_SCAN_KERNEL)
    ms_per_step = sec / args.steps * 1e3
    qps = nq * args.steps / sec
    # context only: the same steps with every stage bracketed (the breakdown in config.stage_ms)
    # and with no events at all
    sec_stages, stage_all = run(chosen, args.steps, profile=binding.PROFILE_STAGES)
    sec_plain, _ = run(chosen, args.steps, profile=False)
    ix.set_profiling(binding.PROFILE_STAGES)
    dco = ix.dco(nq)
    graph_ms = None
    if args.graph:
        # the same search recorded once as a HIP graph (its own workspace and stream order) and
        # replayed: one launch per step instead of some fifteen
        ix.set_profiling(False)
        g_ids, g_d = torch.empty_like(out_ids), torch.empty_like(out_d)
        gs = torch.cuda.Stream()                        # default priority
        with torch.cuda.stream(gs):
            graph = ix.graph(dq, w.k, chosen, w.refine_k, g_ids, g_d, gs)
            for _ in range(args.warmup):
                graph.launch(gs)
            gs.synchronize()
            t = time.perf_counter()
            for _ in range(args.steps):
                graph.launch(gs)
            gs.synchronize()
            graph_ms = (time.perf_counter() - t) / args.steps * 1e3
        same_graph = bool(torch.equal(g_ids, out_ids))
        log(f"[bench] HIP graph replay: {graph_ms:.4f} ms/step against {sec_plain / args.steps * 1e3:.4f} eager; "
            f"ids identical to the eager search: {same_graph}")
        assert same_graph, "the graph's results differ from the eager search"
        graph.free()
    scan_bytes = float(dco.sum()) * (w.M // 2)         # algorithmic: M/2 code bytes per item scored
    scan_gbs = scan_bytes / (stage_all["scan"] * 1e-3) / 1e9
    log(f"[bench] nprobe={chosen} recall@10={rec_chosen} {qps:.0f} QPS, {ms_per_step:.3f} ms/step, "
        f"scan kernel {stage['scan_kernel']:.4f} ms; with all stage events {sec_stages / args.steps * 1e3:.3f} ms/step: "
        f"{stage_all}, scan stage {scan_gbs:.1f} GB/s algorithmic")

    # --- CPU baseline: the oracle as it stands, on a bounded sample of the same batch --------
    # Threads: the host's physical cores as lscpu counts them, capped by what this process may
    # use (its CPU affinity and the OpenMP limit the box sets); and one thread, on a smaller sample.
    from oracle import oracle
    ox = oracle.OracleIndex(hx)
    phys = physical_cores()
    allowed = min(oracle.num_threads(), len(os.sched_getaffinity(0)))
    threads = max(1, min(phys, allowed) if phys else allowed)
    ncpu = args.cpu_queries or 200
    oracle.search(ox, queries[:min(16, nq)], w.k, chosen, w.refine_k, nthreads=threads)          # warm
    t = time.perf_counter()
    want = oracle.search(ox, queries[:ncpu], w.k, chosen, w.refine_k, nthreads=threads)
    cpu_sec = time.perf_counter() - t
    if not args.cpu_queries and cpu_sec < 5.0:                                 # aim for ~10-20 s
        ncpu = int(min(nq, ncpu * 12.0 / max(cpu_sec, 1e-3)))
        t = time.perf_counter()
        want = oracle.search(ox, queries[:ncpu], w.k, chosen, w.refine_k, nthreads=threads)
        cpu_sec = time.perf_counter() - t
    same = bool((out_ids.cpu().numpy()[:ncpu] == want.ids).all())
    n1 = max(1, min(ncpu, int(ncpu / cpu_sec * 4.0 / threads)))               # about 4 s on one thread
    t = time.perf_counter()
    oracle.search(ox, queries[:n1], w.k, chosen, w.refine_k, nthreads=1)
    cpu1_sec = time.perf_counter() - t
    log(f"[bench] oracle: {ncpu} queries in {cpu_sec:.2f}s on {threads} threads (lscpu: {phys} physical cores), "
        f"{n1} queries in {cpu1_sec:.2f}s on 1 thread; GPU ids identical on the sample: {same}")

    # What bounds the dominant kernel.  One table lookup is 16 int8 multiply-adds of the one-hot
    # contraction = 32 ops, so the ops the kernel stands for are items x M x 32 (partly filled
    # query tiles and list tails count as lost).  The register-table kernel issues the 2:4-sparse
    # int8 matrix instruction, the LDS-table kernel the dense one: each is priced against the
    # peak of ITS instruction.  The exact kernel does its lookups on the vector units.
    kernel = ix.scan_kernel_name()
    kms = stage["scan_kernel"]
    lookups = float(dco.sum()) * w.M
    if kernel == "scan_exact_kernel":
        bound, unit = "alu", "T lane-ops/s"
        achieved, peak = lookups * 2 / (kms * 1e-3) / 1e12, LANE_OPS_PEAK / 1e12   # a lookup and an add per code
    else:
        bound, unit = "mfma", "POP/s"
        achieved = lookups * 32 / (kms * 1e-3) / 1e15
        peak = MFMA_I8_SPARSE_POPS if kernel == "scan_mfma_kernel" else MFMA_I8_DENSE_POPS
    kernel_gbs = scan_bytes / (kms * 1e-3) / 1e9
    traffic = measured_traffic(w.name, chosen, kernel)
    hbm_gbs = None if traffic is None else traffic / (kms * 1e-3) / 1e9
    result = {
        "metric": "QPS at recall@10>=0.9 (1Mx128, 1 GPU)" if w.name == "sift1m"
                  else f"QPS at recall@10>={args.target_recall} ({w.name}, 1 GPU)",
        "value": round(qps, 1), "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "i8", "data": "synthetic",
        "config": {
            "workload": f"{w.name}: N={w.n} d={w.d} nq={nq} nlist={w.nlist} M={w.M}x4bit k={w.k} "
                        f"refine_k={w.refine_k} strict AIR lambda=0.5 + SEIL",
            "nprobe": chosen, "recall_at_10": rec_chosen,
            "qps_interpolated_at_target_recall": None if qps_interp is None else round(qps_interp, 1),
            "stage_ms": {k: round(v, 4) for k, v in stage_all.items()},
            "ms_per_step_all_stage_events_on": round(sec_stages / args.steps * 1e3, 4),
            "ms_per_step_events_off": round(sec_plain / args.steps * 1e3, 4),
            "dco_per_query": float(dco.mean()), "index_code_bytes": code_bytes,
            "index_total_bytes": total_bytes, "vectors_in_shared_blocks": round(shared_frac, 4),
            "workspace_bytes": ix.workspace_bytes(nq, chosen, w.refine_k),
            "ms_per_step_hip_graph": None if graph_ms is None else round(graph_ms, 4),
            "ids_identical_to_oracle_on_sample": same,
            "scan_stage_algorithmic_GBs": round(scan_gbs, 1),
        },
        # Dominant kernel: the list-major scan.  Its roof is the matrix pipe (issue of the int8
        # matrix instruction it uses), not HBM: a block fetched once serves a tile of 32 queries,
        # so the algorithmic code bytes (M/2 per item scored, after SEIL dedup; context only)
        # exceed what leaves HBM many times over.  achieved = ops the contraction stands for / the
        # kernel's mean launch time over the timed steps (HIP events on the caller's stream).
        # "traffic" = HBM bytes per launch from the tracked rocprofv3 counter summary for this
        # (workload, nprobe), null when that configuration has none; "hbm" prices it against 8 TB/s.
        "roofline": {
            "kernel": kernel, "bound": bound, "achieved": round(achieved, 4), "peak": peak, "unit": unit,
            "frac": round(achieved / peak, 4), "traffic": traffic,
            "avg_launch_ms": round(kms, 4),
            "algorithmic_bytes_per_launch": scan_bytes,
            "algorithmic_GBs": round(kernel_gbs, 1),
            "hbm": None if traffic is None else {
                "bound": "hbm", "achieved": round(hbm_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(hbm_gbs / HBM_PEAK_GBS, 4)},
        },
        "cpu_baseline": {
            "value": round(ncpu / cpu_sec, 1), "unit": "queries/s", "cores": threads,
            "kind": "oracle", "sample": f"first {ncpu} queries of the batch at nprobe={chosen}",
            "physical_cores_lscpu": phys, "value_1_thread": round(n1 / cpu1_sec, 1),
            "sample_1_thread": f"first {n1} queries",
        },
        "sweep": sweep,
    }
    if args.sweep_out:
        with open(args.sweep_out, "w") as f:
            json.dump(result, f, indent=1)
    ix.free()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
