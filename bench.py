#!/usr/bin/env python3
"""Benchmark of the bucket-training hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2] [--no-cpu-baseline]

A step is one batch (B positive edges) through the whole path: negative sampling, gather,
scores, loss, backward, sparse Adagrad.  Edges and partitions are resident in HBM before
the timed region.  Prints one JSON line.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_F32_PEAK_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
VALU_F32_PEAK_TFLOPS = 157.3      # fp32 vector peak: 256 CUs x 64 lanes x 2 (packed) x 2 (fused multiply-add) x 2.4 GHz
HBM_PEAK_GBS = 8000.0             # MI355X HBM3E peak
# HBM bytes per k_chunk_fast launch from the rocprofv3 counter runs summarised in
# profiles/c2_hbm_traffic.txt (FETCH_SIZE x 2.00 + WRITE_SIZE x 1.00, in KiB, calibrated on a copy)
CHUNK_TRAFFIC_BYTES = {"c2": int((281764.5 * 2.0 + 447782.4) * 1024)}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def run_epochs(args, w, buckets, node, rel, L, graphs, torch) -> int:
    """Whole epochs in the paper's bucket order, partitions staged through the HBM buffer."""
    n = w.num_partitions
    capacity = args.capacity if args.capacity else n
    uses_rel = w.score != graphs.SCORE_DOT
    cfg = L.make_config(num_nodes=w.num_nodes, dim=w.dim, num_partitions=n, buffer_capacity=capacity,
                        num_relations=w.num_relations, score=w.score, loss=w.loss, corrupt=w.corrupt,
                        batch_size=w.batch_size, chunk_size=w.chunk_size, num_negs=w.num_negs,
                        num_degree_negs=w.num_degree_negs, lr=w.lr, eps=w.eps, seed=args.seed,
                        update_mode=L.UPDATE_ATOMIC if args.update_mode == "atomic" else L.UPDATE_DETERMINISTIC)
    ctx = L.legend_init_partitions(cfg, node, rel if uses_rel else None)
    log("[bench] context ready")
    K, W = max(args.steps, 1), args.warmup
    stats = None
    # where the caller keeps the edge list: device (default: a 288 GB card holds it next to the
    # partition buffer; uploaded once, before the timed region), pinned host memory, or pageable
    # host memory (each bucket's edges then cross PCIe inside the timed region)
    edges_mem, keep = L.MEM_HOST, {}
    if args.edges == "device":
        t_up = time.time()
        for key in list(buckets.keys()):
            t = torch.from_numpy(buckets[key]).cuda()
            keep[key] = t
            buckets[key] = (t.data_ptr(), t.shape[0])
        torch.cuda.synchronize()
        edges_mem = L.MEM_DEVICE
        log(f"[bench] bucket edges uploaded to the device in {time.time() - t_up:.1f}s")
    elif args.edges == "pinned":
        t_pin = time.time()
        try:
            for key in list(buckets.keys()):
                e = buckets[key]
                t = torch.empty(e.shape, dtype=torch.int32, pin_memory=True)
                t.numpy()[...] = e
                keep[key] = t
                buckets[key] = t.numpy()
            log(f"[bench] bucket edges copied into pinned host memory in {time.time() - t_pin:.1f}s")
        except RuntimeError as err:             # the box limits pinned memory: the rest stays pageable
            log(f"[bench] pinned {len(keep)} of {len(buckets)} bucket edge arrays, the rest stays pageable ({str(err).splitlines()[0]})")
    for ep in range(W):
        L.legend_train_epoch(ctx, n, buckets, edges_mem=edges_mem, epoch=ep, overlap=not args.no_overlap)
        log(f"[bench] warm-up epoch {ep + 1}/{W} done")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    edges = 0
    for ep in range(W, W + K):
        stats = L.legend_train_epoch(ctx, n, buckets, edges_mem=edges_mem, epoch=ep, overlap=not args.no_overlap)
        edges += stats["edges"]
        log(f"[bench] epoch {ep - W + 1}/{K} done after {time.perf_counter() - t0:.1f}s")
    L.legend_sync(ctx)
    wall = time.perf_counter() - t0
    log(f"[bench] {K} epoch(s), prefetch {'off' if args.no_overlap else 'on'}: {wall:.2f} s, {edges / wall:.3e} edges/s")
    ablation = None
    if args.ablation and not args.no_overlap:
        # the same epochs again with every swap serialised (the paper's "without prefetching")
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        edges2 = 0
        for ep in range(W + K, W + 2 * K):
            edges2 += L.legend_train_epoch(ctx, n, buckets, edges_mem=edges_mem, epoch=ep, overlap=False)["edges"]
        L.legend_sync(ctx)
        wall2 = time.perf_counter() - t1
        log(f"[bench] {K} epoch(s), prefetch off: {wall2:.2f} s, {edges2 / wall2:.3e} edges/s")
        ablation = {"prefetch_off_value": round(edges2 / wall2, 1), "prefetch_off_s_per_epoch": round(wall2 / K, 3),
                    "prefetch_on_s_per_epoch": round(wall / K, 3)}
    out = {
        "metric": "edges/sec trained (1 GPU)", "value": round(edges / wall, 1), "unit": "edges/s", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": round(wall * 1e3 / K, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name} ({w.stands_for}): {w.num_nodes} nodes, {w.num_edges} edges, d={w.dim}, "
                               f"{n} partitions, B={w.batch_size}, C={w.chunk_size}, N={w.num_negs}, sides={w.sides}, "
                               f"score={['dot', 'distmult', 'complex', 'transe-l1'][w.score]}; one step = one epoch, edge list in "
                               f"{args.edges} memory",
                   "update_mode": args.update_mode, "resident_partitions": capacity,
                   "prefetch": not args.no_overlap},
        "fallback_chunks": L.legend_fallback_chunks_read(ctx),
        "epoch": {"batches": stats["batches"], "swaps": stats["swaps"], "buffer_states": stats["buffer_states"],
                  "bytes_per_swap": stats["bytes_per_swap"], "loss_sum": stats["loss_sum"]},
    }
    if ablation:
        out["prefetch_ablation"] = ablation
    L.legend_destroy(ctx)
    print(json.dumps(out), flush=True)
    return 0


def run_rank(args, w, L, graphs, torch, np) -> int:
    """Ranking throughput (Sec. 7 "Metrics"): K calls of legend_rank_edges per corrupted side over a fixed
    set of synthetic test triples, every partition resident."""
    n = w.num_partitions
    node, rel = graphs.init_tables(w, args.seed)
    node *= 300.0
    rel = rel * 300.0 + np.float32(0.5)
    uses_rel = w.score != graphs.SCORE_DOT
    cfg = L.make_config(num_nodes=w.num_nodes, dim=w.dim, num_partitions=n, buffer_capacity=n,
                        num_relations=w.num_relations, score=w.score, loss=w.loss, corrupt=w.corrupt,
                        batch_size=w.batch_size, chunk_size=w.chunk_size, num_negs=w.num_negs,
                        num_degree_negs=w.num_degree_negs, seed=args.seed)
    ctx = L.legend_init_partitions(cfg, node, rel if uses_rel else None)
    for p in range(n):
        L.legend_swap_partition(ctx, -1, p)
    L.legend_sync(ctx)
    rng = np.random.default_rng(args.seed)
    m = args.rank_triples
    src = rng.integers(0, w.num_nodes, m)
    dst = rng.integers(0, w.num_nodes, m)
    r = rng.integers(0, max(w.num_relations, 1), m).astype(np.int32) if uses_rel else None
    cand = None if args.rank_candidates == 0 else rng.integers(0, w.num_nodes, args.rank_candidates)
    n_cand = w.num_nodes if cand is None else len(cand)
    sides = [L.CORRUPT_DST, L.CORRUPT_SRC] if w.corrupt == graphs.CORRUPT_BOTH else [L.CORRUPT_DST]
    K, W = args.steps, args.warmup
    for _ in range(W):
        for side in sides:
            L.legend_rank_edges(ctx, src, r, dst, side, cand)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    dev_ms = 0.0
    for _ in range(K):
        for side in sides:
            g, q, mt = L.legend_rank_edges(ctx, src, r, dst, side, cand)
            dev_ms += mt["ms"]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    flops = 2.0 * m * n_cand * w.dim
    launch_ms = dev_ms / (K * len(sides))
    log(f"[bench] rank: {K} steps, wall {wall * 1e3:.1f} ms, device {dev_ms:.1f} ms, MRR {mt['mrr']:.4f}")
    out = {
        "metric": "test triples ranked/sec (1 GPU)", "value": round(m * K / wall, 1), "unit": "triples/s", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": round(wall * 1e3 / K, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name} ({w.stands_for}) ranking: {m} test triples against {n_cand} candidates "
                               f"({'every node' if cand is None else 'a shared uniform sample'}), {len(sides)} side(s) per step, "
                               f"d={w.dim}, score={['dot', 'distmult', 'complex', 'transe-l1'][w.score]}; ids cross PCIe in, counts out, "
                               f"inside the timed region"},
        "candidate_scores_per_s": round(m * n_cand * len(sides) * K / wall, 1),
        "roofline": {"kernel": "k_rank (gather + scores + compare-and-count, fp32 MFMA)", "bound": "mfma",
                     "achieved": round(flops / (launch_ms * 1e-3) / 1e12, 3), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(flops / (launch_ms * 1e-3) / 1e12 / MFMA_F32_PEAK_TFLOPS, 4), "traffic": None,
                     "flops_per_launch": int(flops), "avg_launch_ms": round(launch_ms, 4)},
    }
    if w.score == graphs.SCORE_TRANSE_L1:
        # a subtraction and a |.|-add per component and pair: vector operations that are not fused multiply-adds
        out["roofline"].update({"kernel": "k_rank_trans (gather + L1 scores + compare-and-count, vector ALU)", "bound": "alu",
                                "peak": VALU_F32_PEAK_TFLOPS / 2,
                                "frac": round(flops / (launch_ms * 1e-3) / 1e12 / (VALU_F32_PEAK_TFLOPS / 2), 4)})
    if not args.no_cpu_baseline:
        from oracle import rank as orank
        t1 = time.perf_counter()
        done = 0
        while done < min(m, 4) or (time.perf_counter() - t1 < 10 and done < m):
            e = slice(done, done + 1)
            orank.rank_counts(w.score, node, rel if uses_rel else None, src[e], None if r is None else r[e], dst[e],
                              orank.SIDE_DST, cand)
            done += 1
        cpu_s = time.perf_counter() - t1
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        out["cpu_baseline"] = {"value": round(done / cpu_s / len(sides), 1), "unit": "triples/s", "cores": cores,
                               "kind": "oracle", "sample": f"{done} of the same triples against the same candidates, one side "
                               f"timed and scaled to {len(sides)}, numpy float64, {cpu_s:.1f} s"}
    L.legend_destroy(ctx)
    print(json.dumps(out), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 200 batches; with --epoch a step is an epoch: 1)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default 20 batches; with --epoch 0)")
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--scale", type=int, default=1, help="divide nodes and edges of the workload (for quick checks)")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batches", type=int, default=1)
    ap.add_argument("--profile-only", action="store_true", help="skip the CPU baseline and the per-kernel pass")
    ap.add_argument("--update-mode", choices=["deterministic", "atomic"], default="deterministic")
    ap.add_argument("--epoch", action="store_true",
                    help="time whole epochs through legend_train_epoch (the paper's bucket order, partition swaps) "
                         "instead of K resident batches; --steps then counts epochs")
    ap.add_argument("--capacity", type=int, default=0, help="buffer slots for --epoch (0: all partitions resident)")
    ap.add_argument("--no-overlap", action="store_true", help="--epoch: serialize swaps (the paper's 'without prefetching')")
    ap.add_argument("--ablation", action="store_true", help="--epoch: afterwards run the same number of epochs with swaps serialised")
    ap.add_argument("--edges", choices=["device", "pinned", "pageable"], default="device",
                    help="--epoch: where the bucket edge arrays live (host arrays cross PCIe bucket by bucket inside the timed region)")
    ap.add_argument("--rank", action="store_true",
                    help="time legend_rank_edges (ranks for MRR / Hits@k) instead of training; a step ranks "
                         "--rank-triples triples on every corrupted side of the workload")
    ap.add_argument("--rank-triples", type=int, default=10_000)
    ap.add_argument("--rank-candidates", type=int, default=0, help="--rank: size of the shared candidate sample (0: every node)")
    ap.add_argument("--dim", type=int, default=0, help="override the embedding dimension of the workload (dimension sweep)")
    ap.add_argument("--score", choices=["dot", "distmult", "complex", "transe"], default=None, help="override the score function")
    ap.add_argument("--batch-size", type=int, default=0, help="override the batch size")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = 1 if args.epoch else 200
    if args.warmup is None:
        args.warmup = 0 if args.epoch else 20
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
        return 2

    import numpy as np
    import torch

    from paper_2505_09258_amd import binding as L
    from workloads import graphs

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 2
    w = graphs.WORKLOADS[args.workload]
    if args.scale > 1:
        w = graphs.scaled(w, args.scale)
    over = {}
    if args.dim:
        over["dim"] = args.dim
    if args.score:
        over["score"] = {"dot": graphs.SCORE_DOT, "distmult": graphs.SCORE_DISTMULT, "complex": graphs.SCORE_COMPLEX,
                         "transe": graphs.SCORE_TRANSE_L1}[args.score]
        if over["score"] != graphs.SCORE_DOT and w.num_relations == 0:
            over["num_relations"] = 1
    if args.batch_size:
        over["batch_size"] = args.batch_size
    if over:
        import dataclasses
        w = dataclasses.replace(w, name=w.name + "+" + ",".join(f"{k}={v}" for k, v in over.items()), **over)

    if args.rank:
        torch.cuda.set_device(0)
        return run_rank(args, w, L, graphs, torch, np)

    t0 = time.time()
    last = [time.time()]

    def progress(what):
        def cb(done, total):
            if time.time() - last[0] > 30:          # a long generation keeps reporting
                last[0] = time.time()
                log(f"[bench] {what}: {done}/{total} after {time.time() - t0:.0f}s")
        return cb

    src, rel_ids, dst = graphs.generate_edges(w, args.seed, progress=progress("edges"))
    buckets = graphs.bucket_edges(w, src, rel_ids, dst, progress=progress("buckets"))
    del src, rel_ids, dst
    log(f"[bench] edges bucketed after {time.time() - t0:.1f}s")
    node, rel = graphs.init_tables(w, args.seed)
    log(f"[bench] generated {w.name}: {w.num_nodes} nodes, {w.num_edges} edges, {len(buckets)} buckets in {time.time() - t0:.1f}s")

    torch.cuda.set_device(0)
    if args.epoch:
        return run_epochs(args, w, buckets, node, rel, L, graphs, torch)
    stream = torch.cuda.Stream()
    n = w.num_partitions
    capacity = n if 2 * w.num_nodes * w.dim * 4 < 64e9 else 3
    cfg = L.make_config(num_nodes=w.num_nodes, dim=w.dim, num_partitions=n, buffer_capacity=capacity,
                        num_relations=w.num_relations, score=w.score, loss=w.loss, corrupt=w.corrupt,
                        batch_size=w.batch_size, chunk_size=w.chunk_size, num_negs=w.num_negs,
                        num_degree_negs=w.num_degree_negs, lr=w.lr, eps=w.eps, seed=args.seed,
                        update_mode=L.UPDATE_ATOMIC if args.update_mode == "atomic" else L.UPDATE_DETERMINISTIC,
                        compute_stream=stream.cuda_stream)
    uses_rel = w.score != graphs.SCORE_DOT
    ctx = L.legend_init_partitions(cfg, node, rel if uses_rel else None)
    log(f"[bench] context ready after {time.time() - t0:.1f}s")
    B = w.batch_size
    K, W = args.steps, args.warmup

    # bucket order of the paper's planner; all partitions of the chosen buckets resident
    states, order, begin, overlap = L.legend_plan_order(n)
    if capacity == n:
        for p in range(n):
            L.legend_swap_partition(ctx, -1, p)
        seq = [tuple(map(int, b)) for b in order]
    else:
        for p in states[0]:
            L.legend_swap_partition(ctx, -1, int(p))
        seq = [tuple(map(int, b)) for b in order[begin[0]:begin[1]]]

    # work list: (bucket, first batch, last batch) covering W then K full batches
    work, need, first_timed = [], W + K, None
    dev_edges = {}
    for (i, j) in seq:
        e = buckets[(i, j)]
        full = e.shape[0] // B
        if full == 0:
            continue
        dev_edges[(i, j)] = torch.from_numpy(e).cuda()
        b = 0
        while b < full and need > 0:
            if need > K:                      # still in warm-up
                take = min(full - b, need - K)
            else:
                take = min(full - b, need)
                if first_timed is None:
                    first_timed = len(work)
            work.append((i, j, b, b + take))
            b += take
            need -= take
        if need == 0:
            break
    if need > 0:
        log(f"[bench] workload has too few full batches for {W}+{K} steps")
        return 2
    torch.cuda.synchronize()

    def run(items):
        for (i, j, b0, b1) in items:
            t = dev_edges[(i, j)]
            L.legend_train_bucket_range(ctx, i, j, t.data_ptr(), m=t.shape[0], edges_mem=L.MEM_DEVICE, epoch=0,
                                        batch_begin=b0, batch_end=b1, want_stats=False)

    names = []
    k = 0
    while L.legend_profile_name(k) is not None:
        names.append(L.legend_profile_name(k))
        k += 1
    chunk_bit = 1 << names.index("chunk")

    # a plain device copy of known size: the streaming ceiling of this machine, and the kernel the
    # rocprofv3 FETCH_SIZE / WRITE_SIZE counters are calibrated against (1 GiB read + 1 GiB written)
    cal_src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    cal_dst.copy_(cal_src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * cal_src.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del cal_src, cal_dst

    run(work[:first_timed])
    L.legend_sync(ctx)
    L.legend_unique_rows_read(ctx)
    L.legend_profile_enable(ctx, chunk_bit)          # HIP events around the dominant kernel only
    L.legend_profile_read(ctx)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_start = time.perf_counter()
    ev0.record(stream)
    run(work[first_timed:])
    ev1.record(stream)
    L.legend_sync(ctx)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    dev_ms = ev0.elapsed_time(ev1)
    prof = L.legend_profile_read(ctx)
    uniq, nbatches = L.legend_unique_rows_read(ctx)
    assert nbatches == K, (nbatches, K)
    edges_per_s = K * B / wall
    log(f"[bench] {K} steps: wall {wall * 1e3:.1f} ms, device {dev_ms:.1f} ms, {edges_per_s:.3e} edges/s")

    # ---- roofline of the dominant kernel (the fused chunk kernel): three contractions per side
    sides = w.sides
    P, N, d = B, w.num_negs, w.dim
    flops_per_launch = sides * 3 * 2 * P * N * d
    chunk_ms = prof["chunk"]["ms"] / max(prof["chunk"]["launches"], 1)
    achieved_tflops = flops_per_launch / (chunk_ms * 1e-3) / 1e12
    shape = L.legend_batch_shape_of(ctx)
    Q = sides * (-(-P // w.chunk_size)) * N
    u_b = uniq / max(nbatches, 1)
    alg_bytes = 12 * P + 4 * Q + 4 * d * (2 * P + Q) + 16 * d * u_b
    single_sweep = (w.dim == 100 and w.loss == graphs.LOSS_SOFTMAX and w.num_negs <= 1024 and args.update_mode != "atomic"
                    and os.environ.get("LEGEND_NO_FAST_CHUNK") != "1")
    kname = ("k_gemm_compose/scores/rowstats/gq/gneg/chain (one launch each)" if w.dim > 128
             else ("k_chunk_fast" if single_sweep else "k_chunk"))
    roofline = {"kernel": kname + " (gather + scores + loss + backward, fp32 MFMA)", "bound": "mfma",
                "achieved": round(achieved_tflops, 3), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved_tflops / MFMA_F32_PEAK_TFLOPS, 4),
                "traffic": CHUNK_TRAFFIC_BYTES.get(w.name) if single_sweep else None,
                "flops_per_launch": flops_per_launch, "avg_launch_ms": round(chunk_ms, 4)}
    translational = w.score == graphs.SCORE_TRANSE_L1
    if translational:
        # No matrix product: per (positive, negative, component) one subtraction and one |.|-add for the
        # score, and for the backward pass a subtraction, a sign transfer and two accumulations: six
        # vector operations, none of them fused multiply-adds (peak = half the fp32 FMA figure).
        flops_per_launch = sides * 6 * P * N * d
        achieved_tflops = flops_per_launch / (chunk_ms * 1e-3) / 1e12
        roofline = {"kernel": "k_chunk_trans (gather + L1 scores + loss + backward, vector ALU)", "bound": "alu",
                    "achieved": round(achieved_tflops, 3), "peak": VALU_F32_PEAK_TFLOPS / 2, "unit": "TFLOP/s",
                    "frac": round(achieved_tflops / (VALU_F32_PEAK_TFLOPS / 2), 4), "traffic": None,
                    "flops_per_launch": flops_per_launch, "avg_launch_ms": round(chunk_ms, 4)}

    # ---- second pass with every kernel class event-timed (separate from the timed region) ----
    kernels = {}
    if not args.profile_only:
        extra = []
        need2 = min(K, 40)
        for (i, j, b0, b1) in work[first_timed:]:
            take = min(need2, b1 - b0)
            if take <= 0:
                break
            extra.append((i, j, b0, b0 + take))
            need2 -= take
        L.legend_profile_enable(ctx, (1 << len(names)) - 1)
        L.legend_profile_read(ctx)
        L.legend_unique_rows_read(ctx)
        run(extra)
        L.legend_sync(ctx)
        prof2 = L.legend_profile_read(ctx)
        uniq2, nb2 = L.legend_unique_rows_read(ctx)
        L.legend_profile_enable(ctx, 0)
        ub2 = uniq2 / max(nb2, 1)
        for name in names:
            if prof2[name]["launches"]:
                kernels[name] = {"ms_per_batch": round(prof2[name]["ms"] / nb2, 4)}
        if "update" in kernels:
            upd_bytes = 16 * d * ub2                       # read E,S and write E,S of every unique row
            stage_bytes = 4 * d * shape["occurrences"]     # staged gradient rows re-read (overhead, not algorithmic)
            ms = kernels["update"]["ms_per_batch"]
            kernels["update"].update({"bound": "hbm", "algorithmic_GBs": round(upd_bytes / ms / 1e6, 1),
                                      "with_staging_GBs": round((upd_bytes + stage_bytes) / ms / 1e6, 1),
                                      "peak_GBs": HBM_PEAK_GBS, "unique_rows_per_batch": round(ub2)})
        if "chunk" in kernels:
            gather_bytes = 4 * d * (2 * P + Q)
            ms = kernels["chunk"]["ms_per_batch"]
            kernels["chunk"].update({"bound": "alu" if translational else "mfma", "TFLOPs": round(flops_per_launch / ms / 1e9, 2),
                                     "gather_GBs": round(gather_bytes / ms / 1e6, 1)})

    out = {
        "metric": "edges/sec trained (1 GPU)", "value": round(edges_per_s, 1), "unit": "edges/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(wall * 1e3 / K, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name} ({w.stands_for}): {w.num_nodes} nodes, {w.num_edges} edges, d={w.dim}, "
                               f"{n} partitions, B={B}, C={w.chunk_size}, N={w.num_negs} ({w.num_degree_negs} degree-weighted), "
                               f"sides={sides}, score={['dot', 'distmult', 'complex', 'transe-l1'][w.score]}",
                   "update_mode": args.update_mode, "resident_partitions": capacity},
        "device_ms_per_step": round(dev_ms / K, 4),
        "algorithmic_bytes_per_step": int(alg_bytes), "unique_rows_per_step": round(u_b),
        "hbm_GBs_whole_step": round(alg_bytes / (wall / K) / 1e9, 1), "copy_GBs_measured": round(copy_gbs, 1),
        "roofline": roofline, "kernels": kernels, "fallback_chunks": L.legend_fallback_chunks_read(ctx),
    }

    # ---- the oracle, as it stands, on this machine's host cores (a baseline, not the target) ------
    if not args.no_cpu_baseline and not args.profile_only:
        from oracle.bucket import OracleConfig, Tables, train_batch
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        ocfg = OracleConfig.from_workload(w, seed=args.seed)
        tab = Tables(ocfg, node, rel if uses_rel else None)
        (i, j, b0, _) = work[first_timed]
        e = buckets[(i, j)]
        t1 = time.perf_counter()
        nb = 0
        while nb < args.cpu_batches or (time.perf_counter() - t1 < 10 and nb < 8):
            train_batch(tab, i, j, e, b0 + nb, 0)
            nb += 1
        cpu_s = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": round(nb * B / cpu_s, 1), "unit": "edges/s", "cores": cores, "kind": "oracle",
                               "sample": f"{nb} batch(es) of {B} edges of bucket ({i},{j}) of the same workload, "
                                         f"numpy float64, {cpu_s:.1f} s"}
    L.legend_destroy(ctx)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
