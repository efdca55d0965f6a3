#!/usr/bin/env python3
"""Benchmark of the VQ-KAN forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch 1024] [--path auto|gather|mfma]
    python bench.py --config {2,4,5} ...      one of the other configurations as the headline of the line
    python bench.py --sweep                   every configuration, one JSON line each

Headline workload: the two-layer Int8 VQ-KAN head 2048 -> 1024 -> 256 (K = 65,536 per
layer, uint16 idx, fp16 gain/bias, tanh between layers), synthetic seeded
parameters and inputs resident in HBM before the timed region.  A step is one
forward of the whole head over one batch.  The headline `value` is edge
evaluations per second at --batch (default 1024); the same line also carries
the batch-1 figures (edge-evals/s and metadata-stream GB/s), the roofline of
the dominant kernel, the L2 hit rate of that kernel's launch (from the counter
summaries under profiles/), the same head through the dense-coefficient
baseline, the CPU oracle timed on a bounded sample, and a short leg for each of
the other configurations (2, 4 cold and warm, 5) with its own roofline, dense
twin and CPU-oracle figure.  Times are medians over five blocks of --steps steps.

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



def load_profile_facts():
    """Counter figures stored by earlier rocprofv3 runs of this file: every line "@kv key=value ..."
    of the summaries under profiles/.  kind=traffic rows carry fetch_bytes / write_bytes per launch
    (FETCH_SIZE and WRITE_SIZE scaled by a copy of known size), kind=l2 rows tcc_hit / tcc_req.
    They describe the kernels as they were when the summary was written; the summary names its
    command, and a row is only used for the very workload, batch and kernel it was taken on."""
    facts = {}
    pdir = os.path.join(ROOT, "profiles")
    for name in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not name.endswith((".txt", ".md")):
            continue
        for line in open(os.path.join(pdir, name), errors="replace"):
            line = line.strip()
            if not line.startswith("@kv "):
                continue
            kv = dict(tok.split("=", 1) for tok in line[4:].split() if "=" in tok)
            try:
                key = (kv["kind"], kv["workload"], int(kv["batch"]), kv["kernel"])
            except (KeyError, ValueError):
                continue
            kv["source"] = "profiles/" + name
            facts[key] = kv
    return facts


def traffic_of(facts, workload, batch, kernel):
    kv = facts.get(("traffic", workload, int(batch), kernel))
    if not kv:
        return None, None
    return int(float(kv["fetch_bytes"]) + float(kv["write_bytes"])), kv["source"]


def l2_of(facts, workload, batch, kernel):
    kv = facts.get(("l2", workload, int(batch), kernel))
    if not kv:
        return None
    hit, req = float(kv["tcc_hit"]), float(kv["tcc_req"])
    return {"kernel": kernel, "tcc_hit": hit, "tcc_req": req, "hit_rate": hit / max(req, 1.0), "source": kv["source"]}


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
    ap.add_argument("--config", type=int, default=3, choices=[2, 3, 4, 5],
                    help="configuration whose leg is the headline of the line (default 3: the metric's own)")
    ap.add_argument("--only", action="store_true", help="run the --config leg alone (short runs under a profiler)")
    ap.add_argument("--variant", default="", help="leg variant: config 4 cold|warm, config 5 i8|f32")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline run, time every benchmark configuration (one JSON line each)")
    ap.add_argument("--probe-copy", action="store_true",
                    help="also run a 256 MiB device copy three times (known traffic: calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def time_steps(torch, fn, steps, warmup, blocks=5):
    """Seconds per step: the median over `blocks` timed blocks of `steps` steps each, every block
    bracketed by a device synchronisation (a single short block now and then catches a stall)."""
    for s in range(warmup):
        fn(s)
    per = []
    n = warmup
    for _ in range(blocks):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            fn(n + s)
        torch.cuda.synchronize()
        per.append((time.perf_counter() - t0) / steps)
        n += steps
    return sorted(per)[len(per) // 2]


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
    # block-floating-point codebook rows (8-bit mantissas, one exponent byte per row: 12-byte rows)
    for B, paths, prepared in ((1, both[:1], False), (1, both[:1], True), (16, both, False), (1024, both[1:], False)):
        ps = synth.config3_layers("f16", cb_dtype="bfp8")
        vq_rows("config3 shape, block-floating-point codebook", [ps], synth.make_x(3960 + B, B, 2048, "uniform"), paths,
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
    # (batch 64 and 128: one and two batch tiles of the fused kernel, which such a layer keeps up to 128)
    (p5,), x5 = synth.config5("i8", B=128)
    for prepared in (False, True):
        copies = [kb.VQLayer(p5) for _ in range(3)]
        if prepared:
            for L in copies:
                L.prepare()
        cases = [(1, "gather"), (4, "gather"), (16, "gather")]
        if not prepared:
            cases += [(64, "gather"), (64, "mfma"), (128, "gather"), (128, "mfma")]
        for B, pname in cases:
            xd = torch.from_numpy(x5[:B]).cuda()
            pth = kb.KAN_PATH_GATHER if pname == "gather" else kb.KAN_PATH_MFMA
            ws = torch.empty(max(kb.kan_vq_workspace_bytes([[copies[0]]], B, pth), 256), dtype=torch.uint8, device="cuda")
            y = torch.empty((B, p5.n_out), dtype=torch.float32, device="cuda")
            turn = [0]

            def fwd():
                kb.kan_vq_layer_forward(copies[turn[0] % 3], xd, path=pth, ws=ws, y=y)
                turn[0] += 1
            t = wall(fwd, 30)
            print(json.dumps({"workload": "config5 layer 4096->4096 K=262144 i8, 3 copies in turn", "batch": B,
                              "path": pname, "prepared": prepared, "rule": "bspline3",
                              "us_per_forward": round(t * 1e6, 2), "edge_evals_per_s": p5.edges * B / t,
                              "metadata_GBps": p5.metadata_bytes / t / 1e9,
                              "kernel": kb.kan_vq_planned_kernel(copies[0], B, 1, pth)}), flush=True)
        del copies
    heads_p, x = synth.config4(50, 64)
    vq_rows("config4 50 Int8 heads 2048->256->21", heads_p, x, both, 10)
    for variant in ("i8", "f32"):
        ps, x = synth.config5(variant)
        vq_rows("config5 4096->4096 K=262144 " + variant, [ps], x, both[1:], 3)


MAIN_KERNELS = ("kan_gather", "kan_mfma", "kan_fused", "kan_bucket", "kan_column")


def roofline_of(kt, lps, layer_edges, layer_meta, B, facts, workload, extra_param_bytes=0):
    """Roofline object of the dominant kernel of a step.  One batch tile (B <= 64): every parameter
    byte is used once, the launch is a stream over its metadata -> HBM.  Above: the contraction
    dominates -> matrix cores (fp16 operands against the fp16 peak, fp32 operands against the fp32
    one) or, for the vector-ALU kernels, the fp32 vector peak."""
    dom = max((k for k in kt if k.startswith(MAIN_KERNELS)), key=lambda k: kt[k]["avg_us"] * kt[k]["launches"])
    avg_s = kt[dom]["avg_us"] * 1e-6
    edges = per_launch(layer_edges, dom, lps[dom])
    family = dom.split("@")[0]
    is_mfma = family.startswith(("kan_mfma", "kan_fused"))
    traffic, tsrc = traffic_of(facts, workload, B, dom)
    if B > 64:
        flops = edges * (B * FLOP_PER_EDGE_EVAL + FLOP_PER_EDGE_RECON)
        peak = PEAK_F16_MFMA_TFLOPS if (is_mfma and family != "kan_fused_f32") else PEAK_FP32_VECTOR_TFLOPS
        roof = {"bound": "mfma" if is_mfma else "alu", "achieved": flops / avg_s / 1e12, "peak": peak, "unit": "TFLOP/s"}
    else:
        nbytes = per_launch(layer_meta, dom, lps[dom])
        roof = {"bound": "hbm", "achieved": nbytes / avg_s / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s"}
    roof.update({"frac": roof["achieved"] / roof["peak"], "kernel": dom, "avg_launch_us": kt[dom]["avg_us"],
                 "traffic": traffic, "traffic_source": tsrc})
    return roof


def run_leg(kb, torch, sets, x, path, steps, warmup, layer_edges, layer_meta, facts, workload, cold=True):
    """Times head calls over `sets` (parameter sets taken in turn: set s % n at step s).
    layer_edges / layer_meta: per layer, summed over the heads of a call."""
    B = x.shape[0]
    heads0 = sets[0]
    ws_bytes = kb.kan_vq_workspace_bytes(heads0, B, path)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    y = torch.empty((len(heads0), B, heads0[0][-1].n_out), dtype=torch.float32, device="cuda")
    n = len(sets) if cold else 1

    def step(s):
        kb.kan_vq_head_forward(sets[s % n], x, path=path, ws=ws, y=y)

    t = time_steps(torch, step, steps, warmup)
    kt = kernel_times(kb, torch, step, min(steps, 50), warmup)
    n_prof = min(steps, 50)
    lps = {k: v["launches"] / n_prof for k, v in kt.items()}
    ee = sum(layer_edges) * B
    roof = roofline_of(kt, lps, layer_edges, layer_meta, B, facts, workload)
    return {"batch": B, "steps": steps, "ms_per_step": 1e3 * t, "edge_evals_per_s": ee / t,
            "metadata_GBps": sum(layer_meta) / t / 1e9, "parameter_sets_rotated": n,
            "kernels_avg_us": {k: round(v["avg_us"], 3) for k, v in kt.items()},
            "kernels_launches_per_step": lps, "kernel_sequence": list(kt.keys()),
            "planned_kernel_layer1": kb.kan_vq_planned_kernel(heads0[0][0], B, len(heads0), path),
            "dominant": roof["kernel"], "roofline": roof, "l2_hit_rate": l2_of(facts, workload, B, roof["kernel"]),
            "workspace_bytes": ws_bytes}


def two_stream_leg(kb, torch, sets, x, path, steps, warmup, edge_evals):
    """Throughput with two requests in flight: the same steps dealt alternately to two streams of equal
    (default) priority, each with its own workspace and output, so that one step's latency-bound phases
    overlap the other's.  Reported beside the one-stream figures, which stay the headline."""
    B = x.shape[0]
    heads0 = sets[0]
    streams = [torch.cuda.Stream() for _ in range(2)]
    wss = [torch.empty(max(kb.kan_vq_workspace_bytes(heads0, B, path), 256), dtype=torch.uint8, device="cuda") for _ in range(2)]
    ys = [torch.empty((len(heads0), B, heads0[0][-1].n_out), dtype=torch.float32, device="cuda") for _ in range(2)]
    torch.cuda.synchronize()

    def step(s):
        with torch.cuda.stream(streams[s & 1]):
            kb.kan_vq_head_forward(sets[s % len(sets)], x, path=path, ws=wss[s & 1], y=ys[s & 1])

    t = time_steps(torch, step, steps, warmup)
    return {"streams": 2, "ms_per_step": 1e3 * t, "edge_evals_per_s": edge_evals / t}


def dense_leg(kb, torch, dims, n_heads, x, steps, warmup):
    """The same shapes through the dense-coefficient baseline (40 bytes per edge): one
    kan_dense_layer_forward per head and layer, tanh (torch) between the layers.  The time does not
    depend on the coefficient values: seeded normal draws of the reconstructed coefficients' scale."""
    B = x.shape[0]
    gen = torch.Generator(device="cuda").manual_seed(1234)
    coefs = [[torch.randn((i, o, 10), generator=gen, dtype=torch.float32, device="cuda") * 0.03 for (i, o) in dims]
             for _ in range(n_heads)]
    wss = [torch.empty(max(kb.kan_dense_workspace_bytes(i, o, B), 256), dtype=torch.uint8, device="cuda") for (i, o) in dims]
    ys = [torch.empty((B, o), dtype=torch.float32, device="cuda") for (_, o) in dims]

    def step(s):
        for h in range(n_heads):
            a = x
            for l in range(len(dims)):
                kb.kan_dense_layer_forward(coefs[h][l], a, ws=wss[l], y=ys[l])
                a = torch.tanh(ys[l]) if l + 1 < len(dims) else ys[l]

    t = time_steps(torch, step, steps, warmup)
    edges = n_heads * sum(i * o for i, o in dims)
    out = {"ms_per_step": 1e3 * t, "edge_evals_per_s": edges * B / t, "coef_bytes": edges * 40,
           "coef_GBps": edges * 40 / t / 1e9, "kernel_layer1": kb.kan_dense_planned_kernel(dims[0][0], dims[0][1], B),
           "calls_per_step": n_heads * len(dims)}
    del coefs
    torch.cuda.empty_cache()
    return out


def cpu_leg(fn, edge_evals, what, reps=5, budget_s=25.0):
    """The float64 numpy oracle as it stands, timed on the host: median of up to `reps` runs of a
    bounded sample (fewer when the budget of CPU seconds is used up)."""
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    ts = []
    t_all = time.perf_counter()
    for _ in range(reps):
        t0 = time.perf_counter()
        fn()
        ts.append(time.perf_counter() - t0)
        if time.perf_counter() - t_all > budget_s:
            break
    t = sorted(ts)[len(ts) // 2]
    return {"value": edge_evals / t, "unit": "edge-evals/s", "cores": int(threads), "kind": "oracle",
            "sample": f"float64 numpy oracle, {what}, median of {len(ts)} ({t:.2f} s each)"}


def leg_config2(kb, torch, synth, args, path, facts, with_cpu, B=16):
    (P,), x = synth.config2(B)
    n_sets = (MALL_BYTES * 5 // 4) // (P.metadata_bytes + P.codebook.nbytes) + 1
    sets = [[[kb.VQLayer(P)]] for _ in range(n_sets)]
    xd = torch.from_numpy(x).cuda()
    r = run_leg(kb, torch, sets, xd, path, args.steps, args.warmup, [P.edges], [P.metadata_bytes], facts, "config2")
    r["workload"] = f"config 2: layer 2048->512, fp32 codebook K=65536, uint16 idx, fp32 gain/bias, batch {B}"
    if not args.only:
        r["dense_baseline"] = dense_leg(kb, torch, [(2048, 512)], 1, xd, args.steps, args.warmup)
    if with_cpu:
        from oracle import kan_oracle as ko
        r["cpu_baseline"] = cpu_leg(lambda: ko.vq_layer_forward(x, **P.as_dict()), P.edges * B, f"the whole layer, batch {B}")
    return r


def leg_config4(kb, torch, synth, args, path, facts, with_cpu, cold=True, n_heads=50, B=64):
    heads_p, x = synth.config4(n_heads, B)
    # cold: two full parameter sets taken in turn (2 x 224 MB, more than the memory-side cache holds)
    sets = [[[kb.VQLayer(p) for p in ps] for ps in heads_p] for _ in range(2 if cold else 1)]
    xd = torch.from_numpy(x).cuda()
    edges = [sum(ps[l].edges for ps in heads_p) for l in range(2)]
    meta = [sum(ps[l].metadata_bytes for ps in heads_p) for l in range(2)]
    r = run_leg(kb, torch, sets, xd, path, args.steps, args.warmup, edges, meta, facts, "config4" if cold else "config4warm", cold=cold)
    r["workload"] = (f"config 4: {n_heads} Int8 heads 2048->256->21 on one shared batch of {B}, one grouped launch per layer, "
                     + ("two parameter sets in turn (cold)" if cold else "one parameter set (cache-warm)"))
    r["codebook_bytes"] = sum(p.codebook.nbytes for ps in heads_p for p in ps)
    if not args.only and cold:
        r["dense_baseline"] = dense_leg(kb, torch, [(2048, 256), (256, 21)], n_heads, xd, max(args.steps // 4, 3), 2)
    if with_cpu and cold:
        from oracle import kan_oracle as ko
        hs = heads_p[:8]
        r["cpu_baseline"] = cpu_leg(lambda: [ko.vq_head_forward(x, [p.as_dict() for p in ps]) for ps in hs],
                                    sum(p.edges for ps in hs for p in ps) * B, f"8 of the {n_heads} heads, whole batch of {B}")
    return r


def leg_config5(kb, torch, synth, args, path, facts, with_cpu, variant="i8", B=8192):
    (P,), x = synth.config5(variant, B=B)
    sets = [[[kb.VQLayer(P)]]]
    xd = torch.from_numpy(x).cuda()
    steps = max(args.steps // 10, 5)
    r = run_leg(kb, torch, sets, xd, path, steps, min(args.warmup, 3), [P.edges], [P.metadata_bytes], facts, "config5_" + variant)
    r["workload"] = (f"config 5: layer 4096->4096, K=262144 {'Int8' if variant == 'i8' else 'fp32'} codebook, uint32 idx, "
                     f"{'fp16' if variant == 'i8' else 'fp32'} gain/bias, batch {B}")
    if not args.only:
        r["dense_baseline"] = dense_leg(kb, torch, [(4096, 4096)], 1, xd, steps, 2)
    if with_cpu:
        from oracle import kan_oracle as ko
        rows = 64
        r["cpu_baseline"] = cpu_leg(lambda: ko.vq_layer_forward(x[:rows], **P.as_dict()), P.edges * rows,
                                    f"the layer on {rows} of the {B} batch rows", reps=3)
    return r


def config3_legs(kb, torch, synth, args, path, facts, with_cpu):
    """The metric's own configuration: batch args.batch and batch 1 (prepared and as given), parameters
    rotated over enough copies to exceed the memory-side cache."""
    layers = synth.config3_layers()
    edges = [p.edges for p in layers]
    meta = [p.metadata_bytes for p in layers]
    param_bytes = sum(meta) + sum(p.codebook.nbytes for p in layers)
    n_copies = args.copies or (MALL_BYTES * 5 // 4 + param_bytes - 1) // param_bytes
    copies = [[kb.VQLayer(p) for p in layers] for _ in range(n_copies)]
    sets = [[cp] for cp in copies]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for cp in copies:
        for L in cp:
            L.prepare()
    torch.cuda.synchronize()
    prepare_ms_per_head = 1e3 * (time.perf_counter() - t0) / len(copies)

    results = {}
    batches = sorted({1, 4, 16, args.batch}) if not args.only else [args.batch]
    legs = [(b, b <= 4 and not args.no_prepare) for b in batches]
    if not args.no_prepare and not args.only:
        legs.append((1, False))
    for B, prepared in legs:
        for cp in copies:
            for L in cp:
                L.use_prepared(prepared)
        steps = args.steps if B > 1 else max(args.steps, 200)
        x = torch.from_numpy(synth.make_x(3900 + B, B, 2048, "uniform")).cuda()
        r = run_leg(kb, torch, sets, x, path, steps, args.warmup, edges, meta, facts, "config3")
        warm = run_leg(kb, torch, sets, x, path, steps, args.warmup, edges, meta, facts, "config3", cold=False) \
            if not args.only else None
        r["prepared_layers"] = bool(prepared)
        if not args.only and B >= 4:
            r["two_streams"] = two_stream_leg(kb, torch, sets, x, path, steps, args.warmup, sum(edges) * B)
        if warm:
            r["ms_per_step_cache_warm"] = warm["ms_per_step"]
            r["edge_evals_per_s_cache_warm"] = warm["edge_evals_per_s"]
        key = B if (prepared or B > 4 or args.no_prepare) else "1_unprepared"
        results[key] = r
    for cp in copies:
        for L in cp:
            L.use_prepared(False)
    B = args.batch
    r = results[B]
    r["workload"] = (f"config 3: two-layer Int8 VQ-KAN head 2048->1024->256, K=65536 per layer, uint16 idx, "
                     f"fp16 gain/bias, tanh between layers, batch {B}")
    if not args.only:
        x = torch.from_numpy(synth.make_x(3900 + B, B, 2048, "uniform")).cuda()
        r["dense_baseline"] = dense_leg(kb, torch, [(2048, 1024), (1024, 256)], 1, x, max(args.steps // 2, 5), 3)
    if with_cpu:
        from oracle import kan_oracle as ko
        rows = min(B, 1024)
        xs = synth.make_x(3900 + B, B, 2048, "uniform")[:rows]
        dl = [p.as_dict() for p in layers]
        ko.vq_head_forward(xs[:8], dl)                       # warm-up (untimed)
        r["cpu_baseline"] = cpu_leg(lambda: ko.vq_head_forward(xs, dl), sum(edges) * rows,
                                    f"whole head on {rows} of the {B} batch rows", reps=11, budget_s=15.0)
    return results, {"parameter_copies_rotated": n_copies, "edges": sum(edges), "metadata_bytes": sum(meta),
                     "prepare_ms_per_head": prepare_ms_per_head}


def dtype_of(r):
    return "f16" if r["roofline"]["kernel"].startswith(("kan_mfma@", "kan_fused_f16")) else "f32"


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one MI355X; runs with --gpus above 1 are not part of this build", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2512_15742_amd import binding as kb
    from paper_2512_15742_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    kb.lib()
    path = {"auto": kb.KAN_PATH_AUTO, "gather": kb.KAN_PATH_GATHER, "mfma": kb.KAN_PATH_MFMA}[args.path]

    if args.sweep:
        sweep(kb, torch, synth)
        return
    facts = load_profile_facts()
    with_cpu = not args.no_cpu_baseline

    if args.probe_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    legs = {}
    extra = {}

    def other(n):          # the legs of the other configurations
        if n == 2:
            return leg_config2(kb, torch, synth, args, path, facts, with_cpu)
        if n == 4:
            cold = args.variant != "warm"
            r = leg_config4(kb, torch, synth, args, path, facts, with_cpu, cold=cold)
            if not args.only and cold:
                w = leg_config4(kb, torch, synth, args, path, facts, False, cold=False)
                r["cache_warm"] = {k: w[k] for k in ("ms_per_step", "edge_evals_per_s", "metadata_GBps", "kernels_avg_us", "roofline")}
            return r
        return leg_config5(kb, torch, synth, args, path, facts, with_cpu, variant=args.variant or "i8")

    if args.config == 3 or not args.only:
        res3, extra = config3_legs(kb, torch, synth, args, path, facts, with_cpu)
        legs[3] = res3[args.batch]
    else:
        res3 = {}
    if args.only:
        if args.config != 3:
            legs[args.config] = other(args.config)
    else:
        for n in (2, 4, 5):
            torch.cuda.empty_cache()
            legs[n] = other(n)

    r = legs[args.config]
    out = {
        "metric": "VQ-KAN edge-evals/sec (Int8 K=65536 head 2048->1024->256)" if args.config == 3
                  else f"VQ-KAN edge-evals/sec (configuration {args.config})",
        "value": r["edge_evals_per_s"], "unit": "edge-evals/s",
        "n_gpus": 1, "steps": r["steps"], "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype_of(r), "data": "synthetic",
        "config": dict({"workload": r["workload"], "batch": r["batch"], "path": args.path}, **extra),
        "metadata_GBps": r["metadata_GBps"],
        "roofline": r["roofline"],
        "l2_hit_rate": r.get("l2_hit_rate"),
        "cpu_baseline": r.get("cpu_baseline"),
        "dense_baseline": r.get("dense_baseline"),
        "timing": "median of 5 blocks of `steps` steps, each block bracketed by a device synchronisation",
    }
    if 3 in legs:
        out["batch%d" % args.batch] = legs[3]
        for b in (1, 4, 16):
            if b in res3 and b != args.batch:
                out["batch%d" % b] = res3[b]
        if "1_unprepared" in res3:
            out["batch1_unprepared"] = res3["1_unprepared"]
        out["prepare_ms_per_head"] = extra.get("prepare_ms_per_head")
    for n in (2, 4, 5):
        if n in legs:
            out["config%d" % n] = legs[n]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
