#!/usr/bin/env python3
"""Benchmark of the VQ-KAN forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch 1024] [--path auto|gather|mfma]

Workload: the two-layer Int8 VQ-KAN head 2048 -> 1024 -> 256 (K = 65,536 per
layer, uint16 idx, fp16 gain/bias, tanh between layers), synthetic seeded
parameters and inputs resident in HBM before the timed region.  A step is one
forward of the whole head over one batch.  The headline `value` is edge
evaluations per second at --batch (default 1024); the same line also carries
the batch-1 figures (edge-evals/s and metadata-stream GB/s), the roofline of
the dominant kernel, and the CPU oracle timed on a bounded sample.

To keep the metadata stream coming from HBM rather than from the 256 MB
memory-side cache, the steps rotate over enough independent parameter copies
to exceed that cache; a second, single-copy ("cache-warm") figure is reported
next to it.
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

PEAK_HBM_GBPS = 8000.0          # MI355X HBM3E
PEAK_FP32_VECTOR_TFLOPS = 157.3
PEAK_F16_MFMA_TFLOPS = 2500.0
FLOP_PER_EDGE_EVAL = 8.0        # 4 multiply-adds under the nonzero cubic bases
FLOP_PER_EDGE_RECON = 20.0      # gain * C[idx] + bias over G = 10, once per launch
MALL_BYTES = 256 << 20

# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc
# (FETCH_SIZE / WRITE_SIZE runs scaled by a copy kernel of known size); see the
# summaries under profiles/.  None until such a run exists for the workload.
MEASURED_TRAFFIC = {
    # bytes per launch (fetched + written) of the layer-1 launch, the dominant one of a step
    ("kan_mfma@L1", 1024): int((60.70 + 32.00) * 2**20),
    ("kan_gather_bt1@L1", 1): int((17.20 + 0.50) * 2**20),
    ("kan_bucket@L1", 1): int((12.93 + 0.03) * 2**20),
}


def layer_of(kernel_key):
    """Timed launches inside a head call are keyed "family@L<layer>" (1-based)."""
    return int(kernel_key.split("@L")[1]) - 1 if "@L" in kernel_key else None


def per_launch(values, kernel_key, launches_per_step):
    """Share of a per-layer quantity (edges, metadata bytes) that one launch of this kernel covers."""
    l = layer_of(kernel_key)
    return (values[l] if l is not None else sum(values)) / launches_per_step


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=1024)
    ap.add_argument("--path", default="auto", choices=["auto", "gather", "mfma"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prepare", action="store_true",
                    help="batch <= 4 on the parameters as given (no kan_vq_prepare regrouping)")
    ap.add_argument("--copies", type=int, default=0, help="parameter copies to rotate over (0 = enough to exceed the memory-side cache)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline run, time every benchmark configuration (one JSON line each)")
    ap.add_argument("--probe-copy", action="store_true",
                    help="also run a 256 MiB device copy three times (known traffic: calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def time_steps(torch, fn, steps, warmup):
    for s in range(warmup):
        fn(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        fn(warmup + s)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def kernel_times(kb, torch, fn, steps, warmup):
    """Average duration per launch of every kernel, HIP events on the launch stream."""
    for s in range(min(warmup, 5)):
        fn(s)
    torch.cuda.synchronize()
    kb.kan_prof_begin(steps * 8)
    for s in range(steps):
        fn(warmup + s)
    torch.cuda.synchronize()
    rec = kb.kan_prof_end()
    return {k: {"launches": v["launches"], "avg_us": 1e3 * v["total_ms"] / max(v["launches"], 1)}
            for k, v in rec.items()}


def run_batch(kb, torch, synth, copies, B, path, steps, warmup, prepared=False):
    for cp in copies:
        for L in cp:
            L.use_prepared(prepared)
    x = torch.from_numpy(synth.make_x(3900 + B, B, 2048, "uniform")).cuda()
    ws_bytes = kb.kan_vq_workspace_bytes([copies[0]], B, path)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    y = torch.empty((1, B, 256), dtype=torch.float32, device="cuda")
    n = len(copies)

    def cold(s):
        kb.kan_vq_head_forward([copies[s % n]], x, path=path, ws=ws, y=y)

    def warm(s):
        kb.kan_vq_head_forward([copies[0]], x, path=path, ws=ws, y=y)

    t_cold = time_steps(torch, cold, steps, warmup)
    t_warm = time_steps(torch, warm, steps, warmup)
    kt = kernel_times(kb, torch, cold, min(steps, 100), warmup)
    return t_cold, t_warm, kt


def sweep(kb, torch, synth):
    """Wall time per forward of every configuration (cache-warm, single parameter copy)."""
    def wall(fn, reps):
        # median of three timed blocks of `reps` calls (a single block now and then catches a stall)
        for _ in range(3):
            fn()
        blocks = []
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            blocks.append((time.perf_counter() - t0) / reps)
        return sorted(blocks)[1]

    def vq_rows(tag, heads_p, x, paths, reps, prepared=False, rule=0):
        heads = [[kb.VQLayer(p, rule=rule) for p in ps] for ps in heads_p]
        if prepared:
            for ls in heads:
                for L in ls:
                    L.prepare()
        xd = torch.from_numpy(x).cuda()
        B = x.shape[0]
        E = sum(p.edges for ps in heads_p for p in ps)
        meta = sum(p.metadata_bytes for ps in heads_p for p in ps)
        for name, path in paths:
            ws = torch.empty(max(kb.kan_vq_workspace_bytes(heads, B, path), 256), dtype=torch.uint8, device="cuda")
            y = torch.empty((len(heads), B, heads_p[0][-1].n_out), dtype=torch.float32, device="cuda")
            t = wall(lambda: kb.kan_vq_head_forward(heads, xd, path=path, ws=ws, y=y), reps)
            print(json.dumps({"workload": tag, "batch": B, "path": name, "prepared": bool(prepared),
                              "rule": "pli2" if rule else "bspline3", "us_per_forward": round(t * 1e6, 2),
                              "edge_evals_per_s": E * B / t, "metadata_GBps": meta / t / 1e9,
                              "kernel": kb.kan_vq_planned_kernel(heads[0][0], B, len(heads), path)}), flush=True)

    both = [("gather", kb.KAN_PATH_GATHER), ("mfma", kb.KAN_PATH_MFMA)]
    ps, x = synth.config1()
    vq_rows("config1 64->32 K=256 fp32", [ps], x, both, 50)
    # the uncompressed twin of config 2: a dense layer of the same shape and value statistics
    # (its time does not depend on the values)
    coef = torch.from_numpy(synth.make_dense_grids(2000, 2048, 512, 65536)[0]).cuda()
    for B in (1, 16, 256, 1024):
        ps, x = synth.config2(B)
        vq_rows("config2 2048->512 K=65536 fp32", [ps], x, both, 30)
        if B == 1:
            vq_rows("config2 2048->512 K=65536 fp32", [ps], x, both[:1], 30, prepared=True)
        xd = torch.from_numpy(x).cuda()
        ws = torch.empty(max(kb.kan_dense_workspace_bytes(2048, 512, B), 256), dtype=torch.uint8, device="cuda")
        y = torch.empty((B, 512), dtype=torch.float32, device="cuda")
        t = wall(lambda: kb.kan_dense_layer_forward(coef, xd, ws=ws, y=y), 30)
        print(json.dumps({"workload": "config2 dense twin 2048x512x10 fp32", "batch": B, "path": "dense",
                          "us_per_forward": round(t * 1e6, 2), "edge_evals_per_s": 2048 * 512 * B / t,
                          "coef_GBps": coef.numel() * 4 / t / 1e9,
                          "kernel": kb.kan_dense_planned_kernel(2048, 512, B)}), flush=True)
    del coef
    for B in (1, 2, 4, 16, 64, 256, 1024, 4096):
        ps, x = synth.config3(B)
        vq_rows("config3 Int8 head 2048->1024->256", [ps], x, both if B <= 1024 else both[1:], 30 if B <= 256 else 10)
        if B <= 4:
            vq_rows("config3 Int8 head 2048->1024->256", [ps], x, both[:1], 30, prepared=True)
    # the runtime operator's two-tap rule on the same head
    for B, paths, prepared in ((1, both[:1], True), (16, both, False), (1024, both[1:], False)):
        ps, x = synth.config3(B)
        vq_rows("config3 Int8 head 2048->1024->256", [ps], x, paths, 30 if B <= 256 else 10, prepared=prepared,
                rule=kb.KAN_RULE_PLI2)
    # the fully quantised 4-bytes-per-edge format (one-byte logarithmic gain, one-byte linear bias)
    for B, paths, prepared in ((1, both[:1], False), (1, both[:1], True), (16, both, False), (1024, both[1:], False)):
        ps = synth.config3_layers("q8")
        vq_rows("config3 shape, 4 B/edge (q8 gain/bias)", [ps], synth.make_x(3900 + B, B, 2048, "uniform"), paths,
                30 if B <= 256 else 10, prepared=prepared)
    # fp16 codebook rows (the middle codebook precision of the paper's Table 1) on the same head
    for B, paths, prepared in ((1, both[:1], False), (1, both[:1], True), (16, both, False), (1024, both[1:], False)):
        ps = synth.config3_layers("f16", cb_dtype="f16")
        vq_rows("config3 shape, fp16 codebook", [ps], synth.make_x(3950 + B, B, 2048, "uniform"), paths,
                30 if B <= 256 else 10, prepared=prepared)
    # residency study: a skewed (trained-like) assignment histogram instead of the uniform worst case
    for dist in ("zipf", "zipf-sorted"):
        for B, paths, prepared in ((1, both[:1], False), (1, both[:1], True), (16, both, False), (1024, both[1:], False)):
            ps = synth.config3_layers("f16", idx_dist=dist)
            vq_rows(f"config3 shape, {dist} idx (s=1)", [ps], synth.make_x(3970 + B, B, 2048, "uniform"), paths,
                    30 if B <= 256 else 10, prepared=prepared)
    # compression side: assign every grid of a dense layer to its nearest codebook shape
    for n_in, n_out, K in ((2048, 1024, 65536), (2048, 512, 65536), (1024, 256, 4096)):
        coef_np, cb_np, _ = synth.make_dense_grids(7000 + K, n_in, n_out, K)
        coef, cb = torch.from_numpy(coef_np).cuda(), torch.from_numpy(cb_np).cuda()
        ws = torch.empty(kb.lib().kan_vq_assign_workspace_bytes(K), dtype=torch.uint8, device="cuda")
        out = kb.kan_vq_assign(coef, cb, ws=ws)
        reps = 3 if K > 10000 else 10
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            out = kb.kan_vq_assign(coef, cb, ws=ws)
        torch.cuda.synchronize()
        t = (time.perf_counter() - t0) / reps
        E = n_in * n_out
        print(json.dumps({"workload": f"assign {n_in}x{n_out} grids to K={K} shapes", "ms": round(t * 1e3, 3),
                          "edges_per_s": E / t, "distances_per_s": E * K / t,
                          "algorithmic_TFLOPs": E * K * 20 / t / 1e12, "issued_mfma_TFLOPs": E * K * 64 / t / 1e12,
                          "r2": kb.kan_vq_reconstruction_r2(coef, cb, *out)}), flush=True)
        del coef, cb
    # a layer large enough to be bandwidth-bound at batch 1: config 5's Int8 layer (134 MB of metadata),
    # three copies taken in turn (402 MB: more than the memory-side cache holds)
    (p5,), x5 = synth.config5("i8", B=16)
    for prepared in (False, True):
        copies = [kb.VQLayer(p5) for _ in range(3)]
        if prepared:
            for L in copies:
                L.prepare()
        for B in (1, 4, 16):
            xd = torch.from_numpy(x5[:B]).cuda()
            pth = kb.KAN_PATH_GATHER
            ws = torch.empty(max(kb.kan_vq_workspace_bytes([[copies[0]]], B, pth), 256), dtype=torch.uint8, device="cuda")
            y = torch.empty((B, p5.n_out), dtype=torch.float32, device="cuda")
            turn = [0]

            def fwd():
                kb.kan_vq_layer_forward(copies[turn[0] % 3], xd, path=pth, ws=ws, y=y)
                turn[0] += 1
            t = wall(fwd, 30)
            print(json.dumps({"workload": "config5 layer 4096->4096 K=262144 i8, 3 copies in turn", "batch": B,
                              "path": "gather", "prepared": prepared, "rule": "bspline3",
                              "us_per_forward": round(t * 1e6, 2), "edge_evals_per_s": p5.edges * B / t,
                              "metadata_GBps": p5.metadata_bytes / t / 1e9,
                              "kernel": kb.kan_vq_planned_kernel(copies[0], B, 1, pth)}), flush=True)
        del copies
    heads_p, x = synth.config4(50, 64)
    vq_rows("config4 50 Int8 heads 2048->256->21", heads_p, x, both, 10)
    for variant in ("i8", "f32"):
        ps, x = synth.config5(variant)
        vq_rows("config5 4096->4096 K=262144 " + variant, [ps], x, both[1:], 3)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one MI355X; runs with --gpus above 1 are not part of this build", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2512_15742_amd import binding as kb
    from paper_2512_15742_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    kb.lib()
    path = {"auto": kb.KAN_PATH_AUTO, "gather": kb.KAN_PATH_GATHER, "mfma": kb.KAN_PATH_MFMA}[args.path]

    if args.sweep:
        sweep(kb, torch, synth)
        return

    layers = synth.config3_layers()
    edges = [p.edges for p in layers]
    meta = [p.metadata_bytes for p in layers]
    param_bytes = sum(meta) + sum(p.codebook.nbytes for p in layers)
    n_copies = args.copies or (MALL_BYTES * 5 // 4 + param_bytes - 1) // param_bytes
    base = [kb.VQLayer(p) for p in layers]
    copies = [base]
    for _ in range(n_copies - 1):           # independent device copies of the same parameters
        cp = []
        for p in layers:
            cp.append(kb.VQLayer(p))
        copies.append(cp)

    if args.probe_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # one-time regrouping of every copy for the small-batch path (kan_vq_prepare), untimed
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for cp in copies:
        for L in cp:
            L.prepare()
    torch.cuda.synchronize()
    prepare_ms_per_head = 1e3 * (time.perf_counter() - t0) / len(copies)

    main_kernels = ("kan_gather", "kan_mfma", "kan_fused", "kan_bucket")
    results = {}
    for B, prepared in [(b, b <= 4 and not args.no_prepare) for b in sorted({1, args.batch})] + \
                       ([] if args.no_prepare else [(1, False)]):
        steps = args.steps if B > 1 else max(args.steps, 500)
        t_cold, t_warm, kt = run_batch(kb, torch, synth, copies, B, path, steps, args.warmup, prepared)
        ee = sum(edges) * B
        dom = max((k for k in kt if k.startswith(main_kernels)),
                  key=lambda k: kt[k]["avg_us"] * kt[k]["launches"])
        key = B if (prepared or B > 4 or args.no_prepare) else "1_unprepared"
        for cp in copies:
            for L in cp:
                L.use_prepared(prepared)
        results[key] = {
            "batch": B, "steps": steps, "prepared_layers": bool(prepared),
            "ms_per_step": 1e3 * t_cold, "edge_evals_per_s": ee / t_cold,
            "metadata_GBps": sum(meta) / t_cold / 1e9,
            "ms_per_step_cache_warm": 1e3 * t_warm, "edge_evals_per_s_cache_warm": ee / t_warm,
            "kernels_avg_us": {k: round(v["avg_us"], 3) for k, v in kt.items()},
            "kernels_launches_per_step": {k: v["launches"] / min(steps, 100) for k, v in kt.items()},
            "planned_kernel_layer1": kb.kan_vq_planned_kernel(base[0], B, 1, path),
            "dominant": dom,
        }

    B = args.batch
    r = results[B]
    dom = r["dominant"]
    # The dominant kernel is one layer's launch (layer 1 here): `achieved` is priced on that
    # layer's edges and on that launch's event-timed duration.
    launches_per_step = r["kernels_launches_per_step"][dom]
    avg_s = r["kernels_avg_us"][dom] * 1e-6
    edges_per_launch = per_launch(edges, dom, launches_per_step)
    family = dom.split("@")[0]
    is_mfma = family.startswith(("kan_mfma", "kan_fused"))
    if B >= 16:
        # compute-bound regime (the metadata stream stops being the limit near B = 12-20)
        flops = edges_per_launch * (B * FLOP_PER_EDGE_EVAL + FLOP_PER_EDGE_RECON)
        # fp16 operands price against the fp16/bf16 matrix-core peak, fp32 operands against the fp32 one
        peak = PEAK_F16_MFMA_TFLOPS if (is_mfma and family != "kan_fused_f32") else PEAK_FP32_VECTOR_TFLOPS
        roof = {"bound": "mfma" if is_mfma else "alu", "achieved": flops / avg_s / 1e12, "peak": peak,
                "unit": "TFLOP/s", "kernel": dom, "avg_launch_us": r["kernels_avg_us"][dom],
                "traffic": MEASURED_TRAFFIC.get((dom, B))}
    else:
        nbytes = per_launch(meta, dom, launches_per_step)
        roof = {"bound": "hbm", "achieved": nbytes / avg_s / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                "kernel": dom, "avg_launch_us": r["kernels_avg_us"][dom],
                "traffic": MEASURED_TRAFFIC.get((dom, B))}
    roof["frac"] = roof["achieved"] / roof["peak"]

    r1 = results[1]
    dom1 = r1["dominant"]
    l1 = r1["kernels_launches_per_step"][dom1]
    roof1 = {"bound": "hbm", "achieved": per_launch(meta, dom1, l1) / (r1["kernels_avg_us"][dom1] * 1e-6) / 1e9,
             "peak": PEAK_HBM_GBPS, "unit": "GB/s", "kernel": dom1, "avg_launch_us": r1["kernels_avg_us"][dom1],
             "traffic": MEASURED_TRAFFIC.get((dom1, 1))}
    roof1["frac"] = roof1["achieved"] / roof1["peak"]
    r1["roofline"] = roof1

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import kan_oracle as ko
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count()
        # a bounded sample: the whole head on the first 1024 rows of the batch (the whole batch of
        # the default run), eleven times: about 10 s of CPU work on a 16-thread host
        rows = min(B, 1024)
        xs = synth.make_x(3900 + B, B, 2048, "uniform")[:rows]
        dl = [p.as_dict() for p in layers]
        ko.vq_head_forward(xs[:8], dl)                       # warm-up (untimed)
        ts = []
        for _ in range(11):
            t0 = time.perf_counter()
            ko.vq_head_forward(xs, dl)
            ts.append(time.perf_counter() - t0)
        t = sorted(ts)[5]
        cpu = {"value": sum(edges) * rows / t, "unit": "edge-evals/s", "cores": int(threads), "kind": "oracle",
               "sample": f"float64 numpy oracle, whole head on {rows} of the {B} batch rows, median of 11 ({t:.2f} s each)"}

    out = {
        "metric": "VQ-KAN edge-evals/sec (Int8 K=65536 head 2048->1024->256)",
        "value": r["edge_evals_per_s"], "unit": "edge-evals/s",
        "n_gpus": 1, "steps": r["steps"], "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if roof["kernel"].startswith(("kan_mfma", "kan_fused_f16")) else "f32", "data": "synthetic",
        "config": {"workload": f"config 3: two-layer Int8 VQ-KAN head 2048->1024->256, K=65536 per layer, "
                               f"uint16 idx, fp16 gain/bias, tanh between layers, batch {B}",
                   "batch": B, "path": args.path, "parameter_copies_rotated": n_copies,
                   "edges": sum(edges), "metadata_bytes": sum(meta)},
        "metadata_GBps": r["metadata_GBps"],
        "roofline": roof,
        "cpu_baseline": cpu,
        "batch1": r1,
        "batch%d" % B: r,
        "prepare_ms_per_head": prepare_ms_per_head,
    }
    if "1_unprepared" in results:
        out["batch1_unprepared"] = results["1_unprepared"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
