#!/usr/bin/env python3
"""Benchmark of the bucket-training hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--no-cpu-baseline] [--per-config none]

A step is one batch (B positive edges) through the whole path: negative sampling, gather,
scores, loss, backward, sparse Adagrad.  Edges and partitions are resident in HBM before
the timed region.  The default workload is c4, the largest single-GPU configuration (Twitter
shape: 41.6 M nodes in 16 partitions behind a three-slot HBM buffer, 1.46 B edges): W + K batches
of the buckets of the first buffer state, in the planner's order.  The same JSON line carries
`per_config`: a short resident-batch run of each other configuration (c1, c2, c3, c5).
Prints one JSON line.
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
# fp32 vector peak of the instructions this build issues (packed fp32 is switched off): 256 CUs x 64 lanes x 2.4 GHz
# = 39.3 T instructions/s; a fused multiply-add counts two operations (78.6 TFLOP/s), anything else one (39.3 T op/s)
VALU_F32_PEAK_TOPS = 39.3
HBM_PEAK_GBS = 8000.0             # MI355X HBM3E peak
# HBM bytes per launch of the dominant kernel and of the update kernel from the rocprofv3 counter runs
# summarised under profiles/ (FETCH_SIZE x 2.00 + WRITE_SIZE x 1.00, in KiB per dispatch, calibrated on a copy)
TRAFFIC_BYTES = {
    "c4": {"source": "profiles/c4_hbm_traffic.txt", "chunk": int((292958.9 * 2.0 + 442406.7) * 1024),
           "update": int((702665.4 * 2.0 + 704152.9) * 1024)},
    "c2": {"source": "profiles/c2_hbm_traffic.txt", "chunk": int((277714.0 * 2.0 + 442328.0) * 1024),
           "update": int((525050.1 * 2.0 + 473205.4) * 1024)},
}


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
                        num_degree_negs=w.num_degree_negs, lr=w.lr, eps=w.eps, seed=args.seed, init_std=w.init_std,
                        update_mode=L.UPDATE_ATOMIC if args.update_mode == "atomic" else L.UPDATE_DETERMINISTIC)
    ctx = L.legend_init_partitions(cfg, node, rel if uses_rel else None)      # node / rel None: the library's seeded fill
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
        "config": {"workload": describe(w, graphs) + f"; one step = one epoch, edge list in {args.edges} memory",
                   "update_mode": args.update_mode, "resident_partitions": capacity,
                   "prefetch": not args.no_overlap},
        "raised_reference_workgroups": L.legend_fallback_chunks_read(ctx),
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
                                "peak": VALU_F32_PEAK_TOPS,
                                "frac": round(flops / (launch_ms * 1e-3) / 1e12 / VALU_F32_PEAK_TOPS, 4)})
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


SCORE_NAMES = ["dot", "distmult", "complex", "transe-l1"]
# graphs above this many edges are not generated whole: only the buckets the run trains are drawn
# (graphs.generate_bucket_edges: the same law, bucket by bucket)
WHOLE_GRAPH_MAX_EDGES = 100_000_000


def describe(w, graphs) -> str:
    return (f"{w.name} ({w.stands_for}): {w.num_nodes} nodes, {w.num_edges} edges, d={w.dim}, {w.num_partitions} partitions, "
            f"B={w.batch_size}, C={w.chunk_size}, N={w.num_negs} ({w.num_degree_negs} degree-weighted), sides={w.sides}, "
            f"score={SCORE_NAMES[w.score]}")


def host_threads() -> int:
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        return os.cpu_count() or 1


def run_resident(args, w, K, W, L, graphs, torch, np, *, kernels_pass=True, cpu_baseline=False, copy_ceiling=True) -> dict:
    """W untimed then K timed batches of workload w with partitions and edges resident in HBM.

    Buckets are taken in the planner's order (Sec. 4) from the first buffer state on; a workload whose
    tables fit comfortably keeps every partition resident, the others get the three-slot buffer and run
    the buckets of the first state.  Returns the measurements as a dict (see main for the JSON line)."""
    t0 = time.time()
    n, B = w.num_partitions, w.batch_size
    uses_rel = w.score != graphs.SCORE_DOT
    table_bytes = 2 * w.num_nodes * w.dim * 4
    capacity = n if (table_bytes < 16e9 or n <= 3) else 3
    states, order, begin, overlap = L.legend_plan_order(n)
    if capacity == n:
        resident = list(range(n))
        seq = [tuple(map(int, b)) for b in order]
    else:
        resident = [int(p) for p in states[0]]
        seq = [tuple(map(int, b)) for b in order[begin[0]:begin[1]]]

    whole = w.num_edges <= WHOLE_GRAPH_MAX_EDGES
    if whole:
        src, rel_ids, dst = graphs.generate_edges(w, args.seed)
        buckets = graphs.bucket_edges(w, src, rel_ids, dst)
        del src, rel_ids, dst
    else:
        # buckets of the run only, enough of them for W + K full batches
        need_edges, wanted = (W + K) * B, []
        expect = w.num_edges / (n * n)
        for b in seq:
            wanted.append(b)
            need_edges -= 0.8 * expect
            if need_edges <= 0:
                break
        buckets, _ = graphs.generate_bucket_edges(w, args.seed, wanted)
        seq = wanted
    log(f"[bench] {w.name}: edges ready after {time.time() - t0:.1f}s ({'whole graph' if whole else f'{len(seq)} buckets of the first buffer state'})")

    stream = torch.cuda.Stream()
    cfg = L.make_config(num_nodes=w.num_nodes, dim=w.dim, num_partitions=n, buffer_capacity=capacity,
                        num_relations=w.num_relations, score=w.score, loss=w.loss, corrupt=w.corrupt,
                        batch_size=B, chunk_size=w.chunk_size, num_negs=w.num_negs,
                        num_degree_negs=w.num_degree_negs, lr=w.lr, eps=w.eps, seed=args.seed, init_std=w.init_std,
                        update_mode=L.UPDATE_ATOMIC if args.update_mode == "atomic" else L.UPDATE_DETERMINISTIC,
                        compute_stream=stream.cuda_stream)
    # initial embeddings: the library's seeded fill, N(0, init_std^2)-like, generated on the device
    ctx = L.legend_init_partitions(cfg, None, None)
    for p in resident:
        L.legend_swap_partition(ctx, -1, p)
    L.legend_sync(ctx)
    log(f"[bench] {w.name}: context ready after {time.time() - t0:.1f}s ({capacity} of {n} partitions resident)")

    # work list: (bucket, first batch, last batch, epoch) covering W then K full batches; a graph with fewer
    # full batches than that (c1, c3) goes round again as the next epoch
    work, need, first_timed = [], W + K, None
    dev_edges = {}
    epoch = 0
    while need > 0:
        before = need
        for (i, j) in seq:
            e = buckets[(i, j)]
            full = e.shape[0] // B
            if full == 0:
                continue
            if (i, j) not in dev_edges:
                dev_edges[(i, j)] = torch.from_numpy(e).cuda()
            b = 0
            while b < full and need > 0:
                if need > K:                      # still in warm-up
                    take = min(full - b, need - K)
                else:
                    take = min(full - b, need)
                    if first_timed is None:
                        first_timed = len(work)
                work.append((i, j, b, b + take, epoch))
                b += take
                need -= take
            if need == 0:
                break
        if need == before or (need > 0 and not whole):
            L.legend_destroy(ctx)
            raise RuntimeError(f"{w.name}: too few full batches in the resident buckets for {W}+{K} steps")
        epoch += 1
    torch.cuda.synchronize()

    def run(items):
        for (i, j, b0, b1, ep) in items:
            t = dev_edges[(i, j)]
            L.legend_train_bucket_range(ctx, i, j, t.data_ptr(), m=t.shape[0], edges_mem=L.MEM_DEVICE, epoch=ep,
                                        batch_begin=b0, batch_end=b1, want_stats=False)

    names = []
    k = 0
    while L.legend_profile_name(k) is not None:
        names.append(L.legend_profile_name(k))
        k += 1
    chunk_bit = 1 << names.index("chunk")

    copy_gbs = None
    if copy_ceiling:
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
    L.legend_fallback_chunks_read(ctx)
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
    fallback = L.legend_fallback_chunks_read(ctx)
    assert nbatches == K, (nbatches, K)
    edges_per_s = K * B / wall
    log(f"[bench] {w.name}: {K} steps: wall {wall * 1e3:.1f} ms, device {dev_ms:.1f} ms, {edges_per_s:.3e} edges/s")

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
    single_sweep = (w.dim in (100, 64) and w.loss == graphs.LOSS_SOFTMAX and w.num_negs <= 1024 and args.update_mode != "atomic"
                    and w.score != graphs.SCORE_TRANSE_L1 and os.environ.get("LEGEND_NO_FAST_CHUNK") != "1")
    kname = ("k_gemm_compose/scores/rowstats/gq/gneg/chain (one launch each)" if w.dim > 128
             else ("k_chunk_fast" if single_sweep else "k_chunk"))
    traffic = TRAFFIC_BYTES.get(w.name.split("+")[0], {})
    roofline = {"kernel": kname + " (gather + scores + loss + backward, fp32 MFMA)", "bound": "mfma",
                "achieved": round(achieved_tflops, 3), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved_tflops / MFMA_F32_PEAK_TFLOPS, 4),
                "traffic": traffic.get("chunk") if single_sweep else None,
                "traffic_source": traffic.get("source") if single_sweep else None,
                "flops_per_launch": flops_per_launch, "avg_launch_ms": round(chunk_ms, 4)}
    translational = w.score == graphs.SCORE_TRANSE_L1
    if translational:
        # No matrix product: per (positive, negative, component) one subtraction and one |.|-add for the
        # score, and for the backward pass a subtraction, a sign transfer and two accumulations: six
        # vector operations, none of them a fused multiply-add (peak: one operation per lane and clock).
        flops_per_launch = sides * 6 * P * N * d
        achieved_tflops = flops_per_launch / (chunk_ms * 1e-3) / 1e12
        roofline = {"kernel": "k_chunk_trans (gather + L1 scores + loss + backward, vector ALU)", "bound": "alu",
                    "achieved": round(achieved_tflops, 3), "peak": VALU_F32_PEAK_TOPS, "unit": "TFLOP/s",
                    "frac": round(achieved_tflops / VALU_F32_PEAK_TOPS, 4), "traffic": None,
                    "flops_per_launch": flops_per_launch, "avg_launch_ms": round(chunk_ms, 4)}

    # ---- second pass with every kernel class event-timed (separate from the timed region) ----
    kernels, update = {}, None
    if kernels_pass:
        extra = []
        need2 = min(K, 40)
        for (i, j, b0, b1, ep) in work[first_timed:]:
            take = min(need2, b1 - b0)
            if take <= 0:
                break
            extra.append((i, j, b0, b0 + take, ep))
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
                # the index side (prepare, sort) runs one batch ahead on its own stream: its figure is a span
                # that contains waiting for compute units, not kernel time
                key = "span_ms_per_batch" if name in ("prepare", "sort") else "ms_per_batch"
                kernels[name] = {key: round(prof2[name]["ms"] / nb2, 4)}
        if "update" in kernels:
            upd_bytes = 16 * d * ub2                       # read E,S and write E,S of every unique row
            stage_bytes = 4 * d * shape["occurrences"]     # staged gradient rows re-read (overhead of the deterministic mode)
            ms = kernels["update"]["ms_per_batch"]
            counter_bytes = traffic.get("update")
            update = {"kernel": "k_update (segmented fp64 sum of the staged gradient rows + Adagrad)", "bound": "hbm",
                      "ms_per_batch": ms, "unique_rows_per_batch": round(ub2),
                      "algorithmic_bytes": int(upd_bytes), "algorithmic_GBs": round(upd_bytes / ms / 1e6, 1),
                      "staged_gradient_bytes": int(stage_bytes),
                      "with_staging_GBs": round((upd_bytes + stage_bytes) / ms / 1e6, 1),
                      "counter_bytes": counter_bytes, "counter_source": traffic.get("source"),
                      "counter_GBs": round(counter_bytes / ms / 1e6, 1) if counter_bytes else None,
                      "peak_GBs": HBM_PEAK_GBS, "frac_of_peak": round(upd_bytes / ms / 1e6 / HBM_PEAK_GBS, 4),
                      "copy_ceiling_GBs": round(copy_gbs, 1) if copy_gbs else None}
            if copy_gbs:
                # what the deterministic design can reach: the kernel must also re-read the staged rows (and, by the
                # counters, over-fetches partial lines of 400-byte rows); at the box's copy rate for all of that,
                # the algorithmic bytes move at this rate
                moved = counter_bytes if counter_bytes else upd_bytes + stage_bytes
                update["structural_ceiling_GBs"] = round(upd_bytes / moved * copy_gbs, 1)
                update["frac_of_structural_ceiling"] = round((upd_bytes / ms / 1e6) / (upd_bytes / moved * copy_gbs), 4)
            kernels["update"].update({"bound": "hbm", "algorithmic_GBs": update["algorithmic_GBs"]})
        if "chunk" in kernels:
            gather_bytes = 4 * d * (2 * P + Q)
            ms = kernels["chunk"]["ms_per_batch"]
            kernels["chunk"].update({"bound": "alu" if translational else "mfma", "TFLOPs": round(flops_per_launch / ms / 1e9, 2),
                                     "gather_GBs": round(gather_bytes / ms / 1e6, 1)})

    res = {
        "workload": w, "value": edges_per_s, "ms_per_step": wall * 1e3 / K, "device_ms_per_step": dev_ms / K,
        "capacity": capacity, "alg_bytes": alg_bytes, "unique_rows": u_b, "copy_gbs": copy_gbs, "roofline": roofline,
        "kernels": kernels, "update": update, "fallback_chunks": fallback, "setup_s": time.time() - t0 - wall,
    }

    # ---- the oracle, as it stands, on this machine's host cores (a baseline, not the target) ------
    if cpu_baseline:
        from oracle.bucket import OracleConfig, Tables, train_batch
        ocfg = OracleConfig.from_workload(w, seed=args.seed)
        (i, j, b0, _, _) = work[first_timed]
        e = buckets[(i, j)]
        rp = w.rows_per_partition
        # the oracle's tables: only the bucket's two partitions, as the GPU holds them now
        tab = Tables.__new__(Tables)
        tab.cfg = ocfg
        tab.E, tab.S = [None] * n, [None] * n
        for p in sorted({i, j}):
            ids = np.arange(p * rp, min(w.num_nodes, (p + 1) * rp), dtype=np.int64)
            tab.E[p] = np.zeros((rp, w.dim), np.float32)
            tab.S[p] = np.zeros((rp, w.dim), np.float32)
            tab.E[p][: ids.size] = L.legend_read_embeddings(ctx, L.TABLE_NODE_EMB, ids, ids.size, w.dim)
            tab.S[p][: ids.size] = L.legend_read_embeddings(ctx, L.TABLE_NODE_STATE, ids, ids.size, w.dim)
        nrel = max(w.num_relations, 1)
        tab.RE = L.legend_read_embeddings(ctx, L.TABLE_REL_EMB, None, nrel, w.dim)
        tab.RS = L.legend_read_embeddings(ctx, L.TABLE_REL_STATE, None, nrel, w.dim)
        t1 = time.perf_counter()
        nb = 0
        while nb < args.cpu_batches or (time.perf_counter() - t1 < 10 and nb < 8):
            train_batch(tab, i, j, e, b0 + nb, 0)
            nb += 1
        cpu_s = time.perf_counter() - t1
        res["cpu_baseline"] = {"value": round(nb * B / cpu_s, 1), "unit": "edges/s", "cores": host_threads(), "kind": "oracle",
                               "sample": f"{nb} batch(es) of {B} edges of bucket ({i},{j}) of the same workload, from the "
                                         f"tables the timed run left, numpy float64, {cpu_s:.1f} s"}
    L.legend_destroy(ctx)
    del dev_edges
    torch.cuda.empty_cache()
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 200 batches; with --epoch a step is an epoch: 1)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default 20 batches; with --epoch 0)")
    ap.add_argument("--workload", default=None, help="c1..c5 (default c4, the largest single-GPU configuration; with --epoch or --rank: c2)")
    ap.add_argument("--scale", type=int, default=1, help="divide nodes and edges of the workload (for quick checks)")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batches", type=int, default=1)
    ap.add_argument("--profile-only", action="store_true", help="skip the CPU baseline, the per-kernel pass and the other configurations")
    ap.add_argument("--per-config", choices=["all", "none"], default=None,
                    help="short resident-batch runs of the other configurations in the same JSON line "
                         "(default: all for the default workload, none when --workload is given)")
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
    default_line = args.workload is None and not (args.epoch or args.rank)
    if args.workload is None:
        args.workload = "c2" if (args.epoch or args.rank) else "c4"
    if args.per_config is None:
        args.per_config = "all" if (default_line and not args.profile_only) else "none"

    import numpy as np
    import torch

    from paper_2505_09258_amd import binding as L
    from workloads import graphs

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 2
    t_all = time.time()
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

    torch.cuda.set_device(0)
    if args.rank:
        return run_rank(args, w, L, graphs, torch, np)

    if args.epoch:
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
        log(f"[bench] generated {w.name}: {w.num_nodes} nodes, {w.num_edges} edges, {len(buckets)} buckets in {time.time() - t0:.1f}s")
        return run_epochs(args, w, buckets, None, None, L, graphs, torch)

    K, W = args.steps, args.warmup
    res = run_resident(args, w, K, W, L, graphs, torch, np, kernels_pass=not args.profile_only,
                       cpu_baseline=not (args.no_cpu_baseline or args.profile_only))
    n = w.num_partitions
    out = {
        "metric": "edges/sec trained (1 GPU)", "value": round(res["value"], 1), "unit": "edges/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(res["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": describe(w, graphs) + (f"; batches of the first buffer state's buckets, {res['capacity']} of {n} "
                                                      f"partitions resident (three-slot buffer)" if res["capacity"] < n else
                                                      "; every partition resident"),
                   "update_mode": args.update_mode, "resident_partitions": res["capacity"]},
        "device_ms_per_step": round(res["device_ms_per_step"], 4),
        "algorithmic_bytes_per_step": int(res["alg_bytes"]), "unique_rows_per_step": round(res["unique_rows"]),
        "hbm_GBs_whole_step": round(res["alg_bytes"] / (res["ms_per_step"] * 1e-3) / 1e9, 1),
        "copy_GBs_measured": round(res["copy_gbs"], 1) if res["copy_gbs"] else None,
        "roofline": res["roofline"], "update": res["update"], "kernels": res["kernels"],
        # workgroups (of K x 1000 x sides) whose single-sweep softmax reference was raised on the way: a tuning aid
        "raised_reference_workgroups": res["fallback_chunks"],
        "update_mode_note": "deterministic is the fast mode: the atomic mode measures 2.1e7 edges/s on c2 against 5.0e7 "
                            "(1.1e8 fp32 atomics per batch cost 1.3 ms, profiles/c2_atomic_kernel_trace.txt)",
    }
    if "cpu_baseline" in res:
        out["cpu_baseline"] = res["cpu_baseline"]

    # ---- the other configurations, each a short resident-batch run (same path, same measurements) ----
    if args.per_config == "all":
        per = {w.name: {"edges_per_s": round(res["value"], 1), "ms_per_batch": round(res["ms_per_step"], 4)}}
        for name, (k2, w2) in {"c1": (300, 20), "c2": (100, 10), "c3": (98, 10), "c5": (60, 10)}.items():
            if name == w.name:
                continue
            if time.time() - t_all > 330:
                per[name] = {"skipped": "time budget of the default run used up"}
                continue
            try:
                r2 = run_resident(args, graphs.WORKLOADS[name], k2, w2, L, graphs, torch, np, kernels_pass=False,
                                  cpu_baseline=False, copy_ceiling=False)
            except Exception as err:            # a configuration that fails does not take the line with it
                per[name] = {"error": str(err).splitlines()[0][:200]}
                continue
            per[name] = {"edges_per_s": round(r2["value"], 1), "ms_per_batch": round(r2["ms_per_step"], 4), "steps": k2,
                         "resident_partitions": r2["capacity"], "dominant_kernel_ms": r2["roofline"]["avg_launch_ms"],
                         "dominant_kernel_frac_of_mfma_peak": r2["roofline"]["frac"],
                         "unique_rows_per_batch": round(r2["unique_rows"]), "raised_reference_workgroups": r2["fallback_chunks"],
                         "workload": describe(graphs.WORKLOADS[name], graphs)}
        out["per_config"] = per
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
