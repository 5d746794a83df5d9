#!/usr/bin/env python3
"""Benchmark of the LoSA prefix-attention hot path on one MI355X.

A "step" is one sparse denoising step (step index >= 1) of ONE layer through losa_step:
locality score + active set, page scoring + top-k + union, paged sparse attention of the
active queries, stable rows reused.  The workload is benchmark configuration C1
(Qwen2.5-7B-like layer, 32k-token prefix, block 32, 20 % active, 2048-token budget).
Consecutive steps rotate over `--layers` independent KV caches (a model's layers), so
every step reads its pages from HBM rather than from the 256 MiB last-level cache.

Prints ONE JSON line.  `value` = microseconds per step per layer (lower is better), inputs
resident in HBM.  `roofline` is for the dominant kernel (the split-K attention kernel, which in
sparse steps also builds the union of the picked pages from the per-row bitmaps while it
starts up): algorithmic bytes (K+V of the pages touched plus the active query rows; the
split-K partials it writes are overhead and not counted) divided by the kernel's mean
duration from HIP events bound to its dispatch, in further passes over the same steps (the
median of three passes is reported).  `cpu_baseline` times the numpy oracle on a sample of
the same steps.  Also reported: dense initialisation (step 0), page-bounds build and in-block
merge times per layer, and the read rate a plain read-only kernel reaches on this GPU over
tiles of the page size, in order and scattered.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=480)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--config", type=int, default=1, help="benchmark configuration index (default C1)")
    ap.add_argument("--layers", type=int, default=16, help="independent KV caches rotated over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of a graph replay")
    ap.add_argument("--warm-single-layer", action="store_true",
                    help="also time the same steps on one layer only (its KV stays cache resident); off by default so "
                         "that a kernel trace of the default run holds cold launches only")
    ap.add_argument("--cpu-steps", type=int, default=12, help="oracle steps timed for cpu_baseline")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: KV load and latency versus the number of active tokens "
                         "and the page budget on configuration C4 (one JSON line per point)")
    ap.add_argument("--calibration-copy-mib", type=int, default=256,
                    help="size of the plain copy launched once as the reference for hardware byte counters")
    ap.add_argument("--read-probe-mib", type=int, default=64,
                    help="bytes per launch of the read-only stream probe over page-sized tiles (0: skip)")
    return ap.parse_args()


def sweep(args):
    """Synthetic analogue of the paper's KV-load-versus-active-tokens figure: configuration C4
    (Llama-3-8B-like, batch 4, 64k prefix, pages of 32, block 64), active fraction in
    {5,10,25,50,100} % x budget in {1024,2048,4096} tokens, plus the dense all-active all-pages
    step.  100 % active is the per-query sparse baseline the paper calls QUEST (Adapted)."""
    import numpy as np
    import torch

    from paper_2604_12056_amd import binding as L
    from paper_2604_12056_amd import synth
    from paper_2604_12056_amd.device_inputs import DeviceBlock, DeviceLayer, config_of

    dev = "cuda:0"
    base = synth.config(4)
    K, V = synth.make_kv(base)
    indptr, indices, total = synth.make_page_table(base)
    lens = np.array(base.seq_lens, dtype=np.int32)
    layer = None
    ctx = L.losa_create(config_of(base, max_topk_pages=4096 // base.g), dev)
    e = 2
    for frac in (0.05, 0.10, 0.25, 0.50, 1.00):
        for budget in (1024, 2048, 4096):
            w = synth.config(4, active_fraction=frac, budget_tokens=budget)
            h, q, picked = synth.make_block_states(w)
            inp = synth.Inputs(w, K, V, h, q, picked, lens, indptr, indices, total)
            if layer is None:
                layer = DeviceLayer(inp, dev)
                L.losa_page_bounds(ctx, layer.kv)
            blk = DeviceBlock(inp, dev)
            mode, param = L.LOSA_SEL_TOPK, float(w.n_active)

            def step(t, diag=None):
                L.losa_step(ctx, layer.kv, t, blk.h[t] if t else None, blk.h[t - 1] if t else None, blk.q[t], mode,
                            param, w.topk_pages, blk.o_p, blk.lse_p, None, diag)

            step(0)
            for t in range(1, w.T):
                step(t)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            step(0)
            e1.record()
            torch.cuda.synchronize()
            dense_us = e0.elapsed_time(e1) * 1e3
            cnt = torch.zeros((w.T, w.batch, w.Hkv), dtype=torch.int32, device=dev)
            reps = 4
            e0.record()
            for _ in range(reps):
                for t in range(1, w.T):
                    step(t, cnt[t])
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / (reps * (w.T - 1))
            pages = cnt[1:].sum(dim=(1, 2)).float().mean().item()
            density = pages / (sum(w.pages_per_seq) * w.Hkv)
            print(json.dumps({"workload": w.name, "active_tokens": w.n_active, "active_fraction": frac,
                              "budget_tokens": budget, "kv_density": round(density, 4),
                              "kv_bytes_per_step": int(pages * w.g * w.d * 2 * e), "sparse_step_us": round(us, 2),
                              "dense_step_us": round(dense_us, 2), "speedup_vs_dense": round(dense_us / us, 2)}),
                  flush=True)
    ctx.close()


def main():
    args = parse_args()
    if args.sweep:
        if args.gpus != 1:
            sys.exit(2)
        return sweep(args)
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only; run with --gpus 1 (no multi-GPU path exists)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2604_12056_amd import binding as L
    from paper_2604_12056_amd import synth
    from paper_2604_12056_amd.device_inputs import DeviceBlock, DeviceLayer, config_of

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    w = synth.config(args.config)
    NL, T = args.layers, w.T
    t0 = time.time()
    inp0 = synth.make_inputs(w)
    layers = [DeviceLayer(inp0, dev)]
    for ell in range(1, NL):
        wl = w.replace(seed=w.seed + 7919 * ell)
        K, V = synth.make_kv(wl)
        layers.append(DeviceLayer(synth.Inputs(wl, K, V, inp0.h, inp0.q, inp0.picked, inp0.seq_lens,
                                               inp0.page_indptr, inp0.page_indices, inp0.num_pages), dev))
    blocks = [DeviceBlock(inp0, dev) for _ in range(NL)]     # per-layer cached (o_p, lse_p)
    ctx = L.losa_create(config_of(w), dev)
    print(f"[bench] {w.name}: {NL} layers generated and uploaded in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    h, q = blocks[0].h, blocks[0].q
    mode, param, topk = L.LOSA_SEL_TOPK, float(w.n_active), w.topk_pages

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---- one plain copy of known size: what FETCH_SIZE / WRITE_SIZE are scaled by under rocprofv3 --pmc
    if args.calibration_copy_mib > 0:
        src = torch.zeros(args.calibration_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        L.losa_calibration_copy(dst, src)
        e0, e1 = ev(), ev()
        e0.record()
        L.losa_calibration_copy(dst, src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbps = 2.0 * src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9      # bytes read + bytes written
        del src, dst
    else:
        copy_gbps = None

    # ---- what a read-only stream over tiles of the page size reaches on this GPU (nothing written):
    # 64 MiB per launch out of a 1 GiB pool (launches about the size of the attention kernel's), tiles in
    # order and in a seeded random order
    read_gbps = {}
    if args.read_probe_mib > 0:
        e_sz = 2 if w.dtype == "bf16" else 4
        tile_bytes = w.g * w.d * e_sz
        pool = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        n_pool = pool.numel() // tile_bytes
        n_read = (args.read_probe_mib << 20) // tile_bytes
        sink = torch.zeros(4096, dtype=torch.uint8, device=dev)
        order = {"linear": torch.arange(n_pool, dtype=torch.int32),
                 "scattered": torch.from_numpy(np.random.Generator(np.random.Philox(4242)).permutation(n_pool).astype(np.int32))}
        for name, ids in order.items():
            ids = ids.to(dev)
            launches = n_pool // n_read
            for rep in range(2):          # the second sweep over the pool is the timed one
                e0, e1 = ev(), ev()
                e0.record()
                for k in range(launches):
                    L.losa_calibration_read(pool, tile_bytes, ids[k * n_read:(k + 1) * n_read], sink)
                e1.record()
                torch.cuda.synchronize()
            read_gbps[name] = launches * n_read * tile_bytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
            # and one launch over the whole pool: the rate without a launch's fixed costs
            e0, e1 = ev(), ev()
            e0.record()
            L.losa_calibration_read(pool, tile_bytes, ids, sink)
            e1.record()
            torch.cuda.synchronize()
            read_gbps[name + "_1GiB_launch"] = n_pool * tile_bytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del pool, sink

    # ---- once per block: page bounds, then the dense initialisation (step 0) of every layer.
    # Each is run eagerly once (results needed below), then timed as one graph replay over all
    # layers so that host launch cost does not count.
    def timed_graph(fn):
        fn()
        torch.cuda.synchronize()
        if args.no_graph:
            e0, e1 = ev(), ev()
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / NL
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / NL

    def all_bounds():
        for ell in range(NL):
            L.losa_page_bounds(ctx, layers[ell].kv)

    def all_dense():
        for ell in range(NL):
            L.losa_step(ctx, layers[ell].kv, 0, None, None, q[0], mode, param, topk, blocks[ell].o_p, blocks[ell].lse_p)

    bounds_us = timed_graph(all_bounds)
    dense_us = timed_graph(all_dense)

    # in-block attention + final merge with the prefix statistics (once per step per layer in a model;
    # reported beside the prefix step, not part of `value`)
    from paper_2604_12056_amd.device_inputs import to_device
    kb, vb = synth.make_block_kv(w)
    dkb, dvb = to_device(kb[1], dev), to_device(vb[1], dev)
    out_full = torch.empty_like(blocks[0].o_p)

    def all_block_merge():
        for ell in range(NL):
            L.losa_block_merge(ctx, q[1], dkb, dvb, blocks[ell].o_p, blocks[ell].lse_p, out_full)

    block_merge_us = timed_graph(all_block_merge)

    # ---- the timed sparse steps
    sel_counts = torch.zeros((args.steps, w.batch, w.Hkv), dtype=torch.int32, device=dev)

    def run_steps(n, first, record=False):
        for i in range(first, first + n):
            ell = i % NL
            t = 1 + (i // NL) % (T - 1)
            L.losa_step(ctx, layers[ell].kv, t, h[t], h[t - 1], q[t], mode, param, topk,
                        blocks[ell].o_p, blocks[ell].lse_p, None, sel_counts[i - first] if record else None)

    run_steps(args.warmup, 0)
    torch.cuda.synchronize()
    # eager launches (one ctypes call per step): host-side launch cost included
    e0, e1 = ev(), ev()
    e0.record()
    run_steps(args.steps, args.warmup)
    e1.record()
    torch.cuda.synchronize()
    eager_us = e0.elapsed_time(e1) * 1e3 / args.steps
    # the same K steps captured once into a HIP graph and replayed: the timed region
    if args.no_graph:
        total_ms, launch = eager_us * args.steps / 1e3, "eager"
    else:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run_steps(args.steps, args.warmup)
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        total_ms, launch = e0.elapsed_time(e1), "hipGraph replay"
    us_per_step = total_ms * 1e3 / args.steps
    # spread over further replays of the same K steps (the reported value stays the first timed replay)
    spread = None
    if not args.no_graph:
        reps = []
        for _ in range(9):
            e0, e1 = ev(), ev()
            e0.record()
            graph.replay()
            e1.record()
            torch.cuda.synchronize()
            reps.append(e0.elapsed_time(e1) * 1e3 / args.steps)
        reps = np.sort(np.array(reps + [us_per_step]))
        spread = {"median": round(float(np.median(reps)), 3), "p10": round(float(np.percentile(reps, 10)), 3),
                  "p90": round(float(np.percentile(reps, 90)), 3), "replays": int(reps.size)}
    warm_us = None
    if not args.no_graph and args.warm_single_layer:
        # the same steps on ONE layer only: its KV stays in the last-level cache between steps (warm figure)
        warm_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(warm_graph):
            for i in range(args.steps):
                t = 1 + i % (T - 1)
                L.losa_step(ctx, layers[0].kv, t, h[t], h[t - 1], q[t], mode, param, topk,
                            blocks[0].o_p, blocks[0].lse_p)
        warm_graph.replay()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        warm_graph.replay()
        e1.record()
        torch.cuda.synchronize()
        warm_us = e0.elapsed_time(e1) * 1e3 / args.steps
        del warm_graph

    # ---- further passes over the same steps with per-kernel events on the launch stream
    # (events bound to a dispatch add packets around it, and how much that stretches a kernel varies
    # from box to box and pass to pass: three passes, the median of their per-stage means is reported)
    passes = []
    for _ in range(3):
        L.losa_profile_enable(ctx, True)
        run_steps(args.steps, args.warmup, record=True)
        torch.cuda.synchronize()
        ms, cnt = L.losa_profile_read(ctx)
        L.losa_profile_enable(ctx, False)
        passes.append({k: (ms[k] * 1e3 / cnt[k] if cnt[k] else None) for k in ms})
    stage_us = {k: (float(np.median([p_[k] for p_ in passes])) if passes[0][k] is not None else None) for k in passes[0]}

    # ---- algorithmic bytes of the attention kernel per launch
    e = 2 if w.dtype == "bf16" else 4
    U = sel_counts.cpu().numpy().astype(np.float64)                    # [steps, batch, Hkv] pages
    pages_per_launch = U.sum(axis=(1, 2)).mean()
    rows = w.batch * w.n_active * w.Hq
    kv_bytes = pages_per_launch * w.g * w.d * 2 * e
    q_bytes = rows * w.d * e
    attn_bytes = kv_bytes + q_bytes                                     # partials are overhead, not counted
    attn_us = stage_us["attn"]
    achieved = attn_bytes / (attn_us * 1e-6) / 1e9
    meta_bytes = sum(w.pages_per_seq) * w.Hkv * 2 * w.d * e
    step_bytes = attn_bytes + meta_bytes + 2 * w.batch * w.B * w.H * e + rows * (w.d + 1) * 4
    density = pages_per_launch / (sum(w.pages_per_seq) * w.Hkv)
    # HBM bytes per launch from hardware counters, if a counter run of this workload was summarised
    traffic = None
    tfile = os.path.join(ROOT, "profiles", f"traffic_{w.name}.txt")
    if os.path.exists(tfile):
        vals = dict(l.split(":", 1) for l in open(tfile) if ":" in l and not l.startswith("#"))
        try:
            traffic = int(float(vals["attn_fetch_bytes_per_launch"]) + float(vals["attn_write_bytes_per_launch"]))
        except (KeyError, ValueError):
            traffic = None

    out = {
        "metric": "sparse-attn us per denoise step per layer (32k prefix)" if args.config == 1
        else "sparse-attn us per denoise step per layer",
        "value": round(us_per_step, 3), "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(total_ms / args.steps, 6), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "q_heads": w.Hq, "kv_heads": w.Hkv, "head_dim": w.d,
                   "prefix_tokens": list(w.seq_lens), "page_size": w.g, "block": w.B, "active_tokens": w.n_active,
                   "budget_pages_per_query": w.topk_pages, "layers_rotated": NL, "denoise_steps": T,
                   "step_kind": "sparse (step index >= 1), full losa_step", "launch": launch},
        "eager_us_per_step": round(eager_us, 3),
        "us_per_step_spread": spread,
        "warm_single_layer_us_per_step": round(warm_us, 3) if warm_us is not None else None,
        "measured_copy_GBps": round(copy_gbps, 1) if copy_gbps is not None else None,
        "measured_read_GBps": {k: round(v, 1) for k, v in read_gbps.items()} or None,
        "step_hbm_GBps": round(step_bytes / (us_per_step * 1e-6) / 1e9, 1),
        "step_bytes": int(step_bytes),
        "union_pages_per_kv_head": round(pages_per_launch / (w.batch * w.Hkv), 1),
        "kv_density": round(float(density), 4),
        "stage_us": {k: (round(v, 3) if v is not None else None) for k, v in stage_us.items()},
        # the same per-kernel figures grouped as the paper's latency breakdown names them (Latency
        # Analysis): reuse for stable tokens is "rows never written", so cache management has no kernel
        "paper_breakdown_us": {
            "locality_pruning": round(stage_us["locality"] or 0.0, 3),
            "criticality_estimation": round((stage_us["score"] or 0.0) + (stage_us["topk"] or 0.0), 3),
            "cache_management": 0.0,
            "attention_computation": round((stage_us["attn"] or 0.0) + (stage_us["merge"] or 0.0), 3)},
        "dense_init_us_per_layer": round(dense_us, 2),
        "dense_init_GBps": round(sum(w.seq_lens) * w.Hkv * w.d * 2 * e / (dense_us * 1e-6) / 1e9, 1),
        # the dense pass is the one place near the matrix-core roof: 4*M*d flop per prefix token and KV head
        # (M = B*G query rows), against 2.5 PFLOP/s dense bf16
        "dense_init_TFLOPs": round(4.0 * w.B * (w.Hq // w.Hkv) * w.d * sum(w.seq_lens) * w.Hkv / (dense_us * 1e-6) / 1e12, 1),
        "dense_init_frac_of_mfma_peak": round(4.0 * w.B * (w.Hq // w.Hkv) * w.d * sum(w.seq_lens) * w.Hkv
                                              / (dense_us * 1e-6) / 2.5e15, 4),
        "block_merge_us_per_layer": round(block_merge_us, 2),
        "page_bounds_us_per_layer": round(bounds_us, 2),
        "page_bounds_GBps": round((sum(w.seq_lens) * w.Hkv * w.d * e + meta_bytes) / (bounds_us * 1e-6) / 1e9, 1),
        "roofline": {"kernel": "attn_mfma_kernel (split-K sparse paged attention; builds the union of the picked pages at start-up)" if w.dtype == "bf16" else "attn_partials_generic_kernel", "bound": "hbm",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_source": (f"profiles/traffic_{w.name}.txt (rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier "
                                        "run of this workload, scaled by the calibration copy; not measured in this run)")
                     if traffic is not None else None,
                     "frac_of_measured_copy": round(achieved / copy_gbps, 4) if copy_gbps else None,
                     "frac_of_measured_scattered_read": round(achieved / read_gbps["scattered"], 4) if read_gbps else None,
                     "bytes_per_launch": int(attn_bytes), "us_per_launch": round(attn_us, 3)},
    }

    if not args.no_cpu_baseline:
        from oracle import losa_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = 1
        cache = orc.PrefixCache(inp0.K, inp0.V, w.g)       # page bounds are built once per block: not timed
        o_ref = np.zeros((w.batch * w.B, w.Hq, w.d)); L_ref = np.zeros((w.batch * w.B, w.Hq))
        n_cpu = min(args.cpu_steps, T - 1)
        c0 = time.perf_counter()
        for t in range(1, 1 + n_cpu):
            orc.losa_step(cache, t, inp0.h[t], inp0.h[t - 1], inp0.q[t], mode, param, topk, w.B, w.Hq, o_ref, L_ref)
        cpu_us = (time.perf_counter() - c0) * 1e6 / n_cpu
        cpu_model = ""
        try:
            with open("/proc/cpuinfo") as f:
                cpu_model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
        except OSError:
            pass
        out["cpu_baseline"] = {"value": round(cpu_us, 1), "unit": "us", "cores": int(cores), "kind": "oracle",
                               "cpu_model": cpu_model, "host_cpus": os.cpu_count(),
                               "sample": f"sparse steps 1..{n_cpu} of layer 0 of {w.name} (numpy float64 oracle)"}
        # the same oracle held to one thread, on fewer steps (reported beside the figure above)
        try:
            from threadpoolctl import threadpool_limits
            n_one = min(4, n_cpu)
            with threadpool_limits(limits=1):
                c0 = time.perf_counter()
                for t in range(1, 1 + n_one):
                    orc.losa_step(cache, t, inp0.h[t], inp0.h[t - 1], inp0.q[t], mode, param, topk, w.B, w.Hq,
                                  o_ref, L_ref)
                out["cpu_baseline"]["single_thread_us"] = round((time.perf_counter() - c0) * 1e6 / n_one, 1)
        except Exception:
            pass
    ctx.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
