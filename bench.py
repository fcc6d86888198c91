#!/usr/bin/env python3
"""Benchmark of the SVOO online stage on one MI355X.

A step = one attention layer of the headline workload (benchmark configs[2]: 12 heads x 75,600
tokens, d = 128, bf16, 256 + 256 clusters, 3 co-clustering iterations, per-layer keep ratio drawn
from [0.08, 0.45]) through the whole hot path: svoo_cocluster -> svoo_permute (Q; K and V) ->
svoo_block_mask -> svoo_block_sparse_attn -> svoo_unpermute, inputs already resident in HBM.
Prints ONE JSON line: whole-layer kept-block TFLOP/s (`value`), ms per layer, the per-call
breakdown, the dense svoo_attn time at the same shape, the roofline fraction of the block-sparse
attention kernel, and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
# Bytes past L2 per svoo_block_sparse_attn launch on configs[2], from the rocprofv3 --pmc passes summarised
# in profiles/sparse_attn_config2_pmc.txt (FETCH_SIZE scaled by 1.97, the factor a copy of known size gives,
# plus WRITE_SIZE); measured offline, at the keep ratios of the first two layers of the sweep.
MEASURED_TRAFFIC_BYTES = {2: 9.8e10}
STEP_NAMES = ("cocluster", "permute", "block_mask", "sparse_attn", "unpermute")


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=12)
    p.add_argument("--warmup", type=int, default=2)
    p.add_argument("--config", type=int, default=2, help="workload id (BASELINE.json configs index)")
    p.add_argument("--inputs", type=int, default=3, help="distinct resident layer inputs cycled through")
    p.add_argument("--mode", default="budget", choices=["budget", "paper"],
                   help="budget: keep ratio alone sets the number of kept blocks (tau=1, theta=0); "
                        "paper: recall 0.95 with switch threshold 0.1")
    p.add_argument("--keep", type=float, default=None, help="fixed keep ratio instead of the per-layer draw")
    p.add_argument("--dense-reps", type=int, default=2)
    p.add_argument("--reuse", type=int, default=20,
                   help="also time one re-clustering period: 1 full step + (reuse-1) steps that keep labels, "
                        "permutations and block lists (0 = skip)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--fused", action="store_true",
                   help="time the four-call path: svoo_block_sparse_attn_tokens folds the Q gather and the "
                        "un-permute into the attention kernel (about 0.6 %% less per layer, but the attention "
                        "launch then also carries the row moves)")
    p.add_argument("--no-density", action="store_true", help="skip the offline attention-density measurement")
    p.add_argument("--density-rows", type=int, default=2048, help="sampled query rows per head for the density")
    p.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of one layer step")
    p.add_argument("--no-microbench", action="store_true",
                   help="skip the matrix-core and copy microbenchmarks the fractions are also quoted against")
    p.add_argument("--no-partitioner-comparison", action="store_true",
                   help="skip the recall comparison of co-clustering against independent k-means")
    p.add_argument("--gen-workers", type=int, default=int(os.environ.get("OMP_NUM_THREADS", "8")))
    return p.parse_args()


def cpu_baseline(cfg, data, keep, tau, theta, scale, kept_flops_layer):
    """The fp64 oracle, as it stands, on one head of the first resident layer end to end: all
    co-clustering iterations at full N, the block mask and block-sparse attention for every query row
    (15-50 s depending on the host); a layer is that times the number of heads (heads are independent
    problems), expressed in the metric's unit."""
    from oracle import svoo_oracle as so
    try:
        from threadpoolctl import threadpool_info
        threads = max([int(x.get("num_threads", 1)) for x in threadpool_info()] + [1])
    except Exception:
        threads = 1
    q, k, v = data["q"][0], data["k"][0], data["v"][0]
    n = q.shape[0]
    t0 = time.perf_counter()
    cc = so.cocluster(q, k, data["init_q_idx"][0], data["init_k_idx"][0], cfg.iters)
    t_cc = time.perf_counter() - t0
    t0 = time.perf_counter()
    mask = so.block_mask(cc["cq"].astype(np.float32).astype(np.float64), cc["ck"].astype(np.float32).astype(np.float64),
                         cc["counts_q"], cc["counts_k"], keep, tau, theta, scale)
    t_mask = time.perf_counter() - t0
    t0 = time.perf_counter()
    so.sparse_attention(q, k, v, cc["labels_q"], cc["labels_k"], mask, scale)
    t_attn = time.perf_counter() - t0
    per_head = t_cc + t_mask + t_attn
    layer_s = per_head * cfg.heads
    return {
        "value": kept_flops_layer / layer_s / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
        "sample": (f"head 0 of layer 0 end to end: {cfg.iters} co-clustering iterations ({t_cc:.1f} s), block mask "
                   f"({t_mask:.2f} s), sparse attention for all {n} query rows ({t_attn:.1f} s) = {per_head:.1f} s/head; "
                   f"x {cfg.heads} heads = {layer_s:.0f} s/layer"),
        "measured_s": per_head, "s_per_head": per_head, "extrapolated_layer_s": layer_s,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (heads are independent problems and would shard across "
              f"GPUs with no collective); --gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_18636_amd import svoo, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    cfg = synth.CONFIGS[args.config]
    dev = "cuda:0"
    tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    scale = float(np.float32(1.0 / math.sqrt(cfg.d)))
    tau, theta = (1.0, 0.0) if args.mode == "budget" else (float(np.float32(0.95)), float(np.float32(0.1)))
    keeps = synth.layer_keeps(cfg) if args.keep is None else np.full(cfg.n_layers, args.keep, dtype=np.float32)

    # ---- resident inputs
    t_gen = time.perf_counter()
    n_inputs = max(1, min(args.inputs, cfg.n_layers))
    host, inputs = [], []
    for layer in range(n_inputs):
        data = synth.make_layer(cfg, layer, workers=args.gen_workers)
        if layer == 0:
            host.append(data)
        inputs.append({key: torch.from_numpy(data[key]).to(dev).to(tdtype if key in "qkv" else torch.int32)
                       for key in ("q", "k", "v", "init_q_idx", "init_k_idx")})
        print(f"[bench] layer input {layer} resident ({time.perf_counter() - t_gen:.1f} s)", file=sys.stderr, flush=True)
    keep_dev = [torch.full((cfg.heads,), float(kp), dtype=torch.float32, device=dev) for kp in keeps]
    layer_obj = svoo.Layer(cfg.heads, cfg.n, cfg.d, tdtype, cfg.kq, cfg.kk, dev)

    def one_step(i, events=None):
        x = inputs[i % n_inputs]
        kp = keep_dev[i % len(keep_dev)]
        if not args.fused:
            calls = (
                # the cluster-order layout comes out of the co-clustering (its last centroid updates sort the
                # labels anyway), so the permute step is the row gather alone
                lambda: layer_obj.step_cocluster_sorted(x["q"], x["k"], x["init_q_idx"], x["init_k_idx"], cfg.iters),
                lambda: layer_obj.step_regather(x["q"], x["k"], x["v"]),
                lambda: layer_obj.step_block_mask(kp, tau, theta, scale),
                lambda: layer_obj.step_attn(scale),
                lambda: layer_obj.step_unpermute(),
            )
        else:   # query-side row moves inside the attention kernel: no Q gather, no separate un-permute launch
            calls = (
                lambda: layer_obj.step_cocluster_sorted(x["q"], x["k"], x["init_q_idx"], x["init_k_idx"], cfg.iters),
                lambda: layer_obj.step_regather_kv(x["k"], x["v"]),
                lambda: layer_obj.step_block_mask(kp, tau, theta, scale),
                lambda: layer_obj.step_attn_fused(x["q"], scale),
                lambda: None,
            )
        for c, call in enumerate(calls):
            if events is not None:
                events[c][0].record()
            call()
            if events is not None:
                events[c][1].record()

    for i in range(args.warmup):
        one_step(i)
        torch.cuda.synchronize()
        print(f"[bench] warm-up step {i} done", file=sys.stderr, flush=True)

    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in STEP_NAMES]
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(i, ev[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    step_ms = np.array([[a.elapsed_time(b) for (a, b) in ev[i]] for i in range(args.steps)])
    print(f"[bench] timed {args.steps} steps: {ms_per_step:.2f} ms/step", file=sys.stderr, flush=True)

    # ---- kept-block work per step (untimed re-run of clustering + mask; results are deterministic)
    kept_flops, phis = [], []
    cache = {}
    for i in range(args.steps):
        key = (i % n_inputs, i % len(keep_dev))
        if key not in cache:
            x = inputs[key[0]]
            layer_obj.step_cocluster(x["q"], x["k"], x["init_q_idx"], x["init_k_idx"], cfg.iters)
            layer_obj.step_block_mask(keep_dev[key[1]], tau, theta, scale)
            nq = layer_obj.counts_q.double()
            nk = layer_obj.counts_k.double()
            pairs = torch.einsum("bq,bqk,bk->", nq, layer_obj.bitmap.double(), nk).item()
            cache[key] = pairs
        pairs = cache[key]
        kept_flops.append(4.0 * cfg.d * pairs)
        phis.append(pairs / (cfg.heads * float(cfg.n) ** 2))
    kept_flops = np.array(kept_flops)
    total_kept = float(kept_flops.sum())

    # ---- dense baseline of this build at the same shape
    x = inputs[0]
    dense_flops = 4.0 * cfg.heads * float(cfg.n) ** 2 * cfg.d
    dense_ms = float("nan")
    if args.dense_reps > 0:
        layer_obj.dense(x["q"], x["k"], x["v"], scale)
        torch.cuda.synchronize()
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        d0.record()
        for _ in range(args.dense_reps):
            layer_obj.dense(x["q"], x["k"], x["v"], scale)
        d1.record()
        torch.cuda.synchronize()
        dense_ms = d0.elapsed_time(d1) / args.dense_reps
        print(f"[bench] dense svoo_attn: {dense_ms:.1f} ms", file=sys.stderr, flush=True)

    # ---- the same layer step recorded once into a HIP graph and replayed (every call only enqueues kernels)
    graph_leg = None
    if not args.no_graph:
        x, kp = inputs[0], keep_dev[0]

        def plain_step():
            layer_obj.run(x["q"], x["k"], x["v"], x["init_q_idx"], x["init_k_idx"], cfg.iters, kp, tau, theta, scale)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            plain_step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        want = layer_obj.out.clone()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            plain_step()
        torch.cuda.synchronize()
        times = {}
        for name, fn in (("eager_ms", plain_step), ("replay_ms", graph.replay)):
            fn()
            torch.cuda.synchronize()
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            g0.record()
            for _ in range(5):
                fn()
            g1.record()
            torch.cuda.synchronize()
            times[name] = round(g0.elapsed_time(g1) / 5, 3)
        graph_leg = {"keep": round(float(keeps[0]), 4), **times,
                     "replay_equals_eager": bool(torch.equal(layer_obj.out, want))}
        del graph
        print(f"[bench] HIP graph: {graph_leg}", file=sys.stderr, flush=True)

    # ---- clustering reuse (paragraph "Clustering Reuse"; the paper re-clusters every 20 diffusion steps)
    reuse = None
    if args.reuse > 1:
        x = inputs[0]
        gen = torch.Generator(device=dev).manual_seed(18636)
        drifted = [tuple((x[key].float() + 0.02 * torch.randn(x[key].shape, device=dev, generator=gen)).to(tdtype)
                         for key in ("q", "k", "v")) for _ in range(2)]
        kp = keep_dev[0]
        layer_obj.run(x["q"], x["k"], x["v"], x["init_q_idx"], x["init_k_idx"], cfg.iters, kp, tau, theta, scale)
        layer_obj.run_reused(*drifted[0], scale)
        torch.cuda.synchronize()
        r0, r1, r2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        r0.record()
        layer_obj.run(x["q"], x["k"], x["v"], x["init_q_idx"], x["init_k_idx"], cfg.iters, kp, tau, theta, scale)
        r1.record()
        for i in range(args.reuse - 1):
            layer_obj.run_reused(*drifted[i % 2], scale)
        r2.record()
        torch.cuda.synchronize()
        full_ms, reused_ms = r0.elapsed_time(r1), r1.elapsed_time(r2) / (args.reuse - 1)
        period_ms = (full_ms + reused_ms * (args.reuse - 1)) / args.reuse
        reuse = {"recluster_every": args.reuse, "keep": round(float(keeps[0]), 4), "full_step_ms": round(full_ms, 3),
                 "reused_step_ms": round(reused_ms, 3), "amortised_ms_per_step": round(period_ms, 3),
                 "amortised_kept_tflops": round(cache[(0, 0)] * 4.0 * cfg.d / (period_ms * 1e-3) / 1e12, 2)
                 if (0, 0) in cache else None}
        print(f"[bench] reuse period of {args.reuse}: {period_ms:.2f} ms/step amortised", file=sys.stderr, flush=True)

    # ---- co-clustering against independent K-means at the same budget (clustering-strategy comparison of
    # the paper, ablation "w/o On"): attention recall = dense softmax mass on kept keys, from the kernels' LSEs
    comparison = None
    if not args.no_partitioner_comparison:
        x = inputs[0]
        kp = torch.full((cfg.heads,), 0.2, dtype=torch.float32, device=dev)
        comparison = {"keep": 0.2, "selection": "budget (tau=1, theta=0)", "layer_input": 0}
        for name, part in (("cocluster", lambda: layer_obj.step_cocluster(x["q"], x["k"], x["init_q_idx"],
                                                                          x["init_k_idx"], cfg.iters)),
                           ("kmeans", lambda: layer_obj.step_kmeans(x["q"], x["k"], x["init_q_idx"], x["init_k_idx"],
                                                                    cfg.iters))):
            part()
            torch.cuda.synchronize()
            p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            p0.record()
            part()
            p1.record()
            layer_obj.step_permute(x["q"], x["k"], x["v"])
            layer_obj.step_block_mask(kp, 1.0, 0.0, scale)
            rec = layer_obj.row_recall(x["q"], x["k"], x["v"], scale)
            torch.cuda.synchronize()
            pairs = torch.einsum("bq,bqk,bk->", layer_obj.counts_q.double(), layer_obj.bitmap.double(),
                                 layer_obj.counts_k.double()).item()
            comparison[name] = {"attention_recall": round(float(rec.double().mean().item()), 4),
                                "kept_fraction": round(pairs / (cfg.heads * float(cfg.n) ** 2), 4),
                                "partition_ms": round(p0.elapsed_time(p1), 3)}
        print(f"[bench] partitioner comparison: {comparison}", file=sys.stderr, flush=True)

    # ---- offline profiling (Sec. 4.1): attention density of layer input 0 on a row sample, tau = 0.95
    density = None
    if not args.no_density:
        x = inputs[0]
        n_rows = min(cfg.n, args.density_rows)
        rows = torch.from_numpy(np.sort(np.random.default_rng(18636).choice(cfg.n, n_rows, replace=False))
                                .astype(np.int32)).to(dev)
        svoo.attention_density(x["q"], x["k"], 0.95, scale, rows=rows)
        torch.cuda.synchronize()
        q0, q1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        q0.record()
        _, dens, passes = svoo.attention_density(x["q"], x["k"], 0.95, scale, rows=rows, want_passes=True)
        q1.record()
        torch.cuda.synchronize()
        d_ms = q0.elapsed_time(q1)
        n_pass = int(passes.max().item())
        density = {"tau": 0.95, "rows_per_head": n_rows, "density_mean": round(float(dens.mean().item()), 5),
                   "density_min": round(float(dens.min().item()), 5), "density_max": round(float(dens.max().item()), 5),
                   "ms": round(d_ms, 3), "passes_max": n_pass,
                   "score_tflops_upper": round(float(passes.double().sum().item()) * 2.0 * n_rows * cfg.n * cfg.d
                                               / (d_ms * 1e-3) / 1e12, 1)}
        print(f"[bench] offline density: {density}", file=sys.stderr, flush=True)

    # ---- what this GPU sustains on the two resources the fractions are quoted against: matrix-core
    # instructions on register operands with nothing else running, and a plain copy of one tensor
    measured = None
    if not args.no_microbench:
        sink = torch.empty((2048 * 256,), dtype=torch.float32, device=dev)
        measured = {}
        for name, rnd in (("mfma_bf16_random_operands_tflops", True), ("mfma_bf16_constant_operands_tflops", False)):
            svoo.microbench_mfma_bf16(sink, 2000, rnd)
            torch.cuda.synchronize()
            m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            m0.record()
            fl = svoo.microbench_mfma_bf16(sink, 20000, rnd)
            m1.record()
            torch.cuda.synchronize()
            measured[name] = round(fl / (m0.elapsed_time(m1) * 1e-3) / 1e12, 1)
        src, dst = inputs[0]["v"], layer_obj.v_sorted
        svoo.microbench_copy(src, dst)
        torch.cuda.synchronize()
        m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        m0.record()
        for _ in range(5):
            moved = svoo.microbench_copy(src, dst)
        m1.record()
        torch.cuda.synchronize()
        measured["copy_GBps"] = round(5 * moved / (m0.elapsed_time(m1) * 1e-3) / 1e9, 1)
        measured["copy_bytes"] = moved
        print(f"[bench] measured peaks: {measured}", file=sys.stderr, flush=True)

    attn_ms = step_ms[:, 3]
    attn_tflops = float(kept_flops.sum() / (attn_ms.sum() * 1e-3) / 1e12)
    value = total_kept / elapsed / 1e12
    result = {
        "metric": "kept-block TFLOPS & ms/layer (cluster+attn), 12h x 75600 tok d128 bf16",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{cfg.cfg_id}] {cfg.name}: {cfg.heads} heads x {cfg.n} tokens "
                               f"(grid {cfg.grid}), d={cfg.d}, {cfg.dtype}, K_q={cfg.kq}, K_k={cfg.kk}, "
                               f"{cfg.iters} co-clustering iterations, per-layer keep from the {cfg.n_layers}-layer "
                               f"draw, selection mode {args.mode} (tau={tau}, theta={theta})",
                   "global_batch": 1, "seq_len": cfg.n, "heads": cfg.heads, "resident_layer_inputs": n_inputs,
                   "keep_mean": round(float(np.mean([keeps[i % len(keeps)] for i in range(args.steps)])), 4)},
        "value_definition": "kept-block FLOPs (4*d*sum over kept blocks of n_r*n_j, true cluster sizes) of all "
                            "timed steps / wall time of the whole layer path",
        "kept_fraction_mean": round(float(np.mean(phis)), 4),
        "breakdown_ms": {name: round(float(step_ms[:, c].mean()), 3) for c, name in enumerate(STEP_NAMES)},
        "path": "five calls (svoo_cocluster_sorted / svoo_gather of Q,K,V / mask / attention / un-permute)"
                if not args.fused else
                "four calls: co-clustering, permute K,V, mask, svoo_block_sparse_attn_tokens (Q gather and "
                "un-permute inside the attention kernel; breakdown_ms.unpermute is therefore 0)",
        "sparse_attn_kept_tflops": round(attn_tflops, 2),
        "dense_attn_ms": round(dense_ms, 2) if args.dense_reps > 0 else None,
        "dense_attn_tflops": round(dense_flops / (dense_ms * 1e-3) / 1e12, 2) if args.dense_reps > 0 else None,
        "speedup_vs_own_dense": round(dense_ms / ms_per_step, 3) if args.dense_reps > 0 else None,
        "roofline": {"bound": "mfma", "kernel": "sparse_attn_bf16_kernel<128, 4, 2>", "achieved": round(attn_tflops, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.cfg_id) if args.keep is None else None,
                     "traffic_note": "bytes past L2 per launch (Infinity Cache + HBM), from rocprofv3 --pmc passes; "
                                     "see profiles/sparse_attn_config2_pmc.txt",
                     "launch_ms": round(float(attn_ms.mean()), 3),
                     "flops_per_launch": float(kept_flops.mean())},
    }
    if reuse is not None:
        result["clustering_reuse"] = reuse
    if comparison is not None:
        result["partitioner_comparison"] = comparison
    if density is not None:
        result["offline_density"] = density
    if graph_leg is not None:
        result["hip_graph"] = graph_leg
    if measured is not None:
        tensor_bytes = cfg.heads * cfg.n * cfg.d * (2 if cfg.dtype == "bf16" else 4)
        perm_ms, unperm_ms = float(step_ms[:, 1].mean()), float(step_ms[:, 4].mean())
        measured["frac_of_measured_mfma"] = round(attn_tflops / measured["mfma_bf16_random_operands_tflops"], 4)
        if not args.fused and unperm_ms > 0:
            measured["row_gather_GBps"] = round(6 * tensor_bytes / (perm_ms * 1e-3) / 1e9, 1)
            measured["unpermute_GBps"] = round(2 * tensor_bytes / (unperm_ms * 1e-3) / 1e9, 1)
        result["measured_peaks"] = measured
    if not args.no_cpu_baseline:
        print("[bench] timing the CPU oracle on a bounded sample ...", file=sys.stderr, flush=True)
        result["cpu_baseline"] = cpu_baseline(cfg, host[0], keeps[0], tau, theta, scale, float(kept_flops[0]))
        result["cpu_baseline"]["value"] = round(result["cpu_baseline"]["value"], 6)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
