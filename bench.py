#!/usr/bin/env python3
"""Benchmark of the compressed-activation convolution training step on one MI355X.

A step is one pass of the whole hot path over one batch of seeded synthetic
input: for every layer of the workload, conv_fwd_and_compress (forward conv +
pooling of the saved input), conv_bwd_weight_compressed (dW from the pooled map)
and conv_bwd_data.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line on stdout; tables go to stderr.
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2_resnet18_cifar")
    ap.add_argument("--layers", default="", help="comma-separated layer indices of the workload (default all)")
    ap.add_argument("--no-graph", action="store_true", help="launch every call from Python instead of a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-backward", action="store_true",
                    help="the step calls conv_bwd_weight_compressed and conv_bwd_data instead of conv_bwd_weight_and_data")
    ap.add_argument("--only", default="", choices=["", "dw", "compress", "fwd", "dx", "copy"],
                    help="profiling aid: run just this entry point --steps times per layer and exit "
                         "(copy: a plain 256 MiB device copy, the yardstick the HBM counters are scaled by)")
    ap.add_argument("--also", default="cfg5_deep_small_spatial",
                    help="second workload whose dW launches are timed too (reported under dw_other_workloads); '' for none")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    return ap.parse_args()


class Layer:
    """Device buffers of one layer of the workload."""

    def __init__(self, spec, config, B, synth, torch, dw_only=False):
        upload = B.to_device
        self.spec = spec
        self.d = B.desc_from_spec(spec)
        hp, wp, self.z_bytes, self.x_bytes = B.cac_pooled_shape(self.d)
        td = torch.float32 if spec.dtype == synth.F32 else torch.bfloat16
        dev = "cuda:0"
        self.ws = {}
        ops = (B.OP_BWD_WEIGHT_COMPRESSED,) if dw_only else (B.OP_FWD_AND_COMPRESS, B.OP_BWD_WEIGHT_COMPRESSED, B.OP_BWD_DATA,
                                                              B.OP_BWD_WEIGHT_AND_DATA)
        for op in ops:
            n = B.cac_workspace_size(self.d, op)
            self.ws[op] = torch.empty(max(n, 16), dtype=torch.uint8, device=dev) if n else None
        self.Z = torch.empty((spec.N, spec.C, hp, wp), dtype=td, device=dev)
        self.dW = torch.empty((spec.K, spec.C, spec.R, spec.S), dtype=torch.float32, device=dev)
        if dw_only:
            # only what the weight gradient reads: Z comes from the library's own compress pass
            t = synth.make_inputs(spec, config, tensors=("X", "dY"))
            X = upload(t["X"], spec.dtype)
            self.dY = upload(t["dY"], spec.dtype)
            B.cac_compress(self.d, X, self.Z, torch.cuda.current_stream())
            torch.cuda.synchronize()
            del X
        else:
            t = synth.make_inputs(spec, config)
            self.X, self.W, self.b, self.dY = (upload(t[k], spec.dtype) for k in ("X", "W", "b", "dY"))
            self.Y = torch.empty((spec.N, spec.K, spec.P, spec.Q), dtype=td, device=dev)
            self.dX = torch.empty((spec.N, spec.C, spec.H, spec.W), dtype=td, device=dev)
        self.plan = B.cac_describe_plan(self.d, B.OP_BWD_WEIGHT_COMPRESSED)
        eb = spec.elem_bytes
        self.flops = {
            "fwd": 2 * spec.N * spec.P * spec.Q * spec.K * spec.C * spec.R * spec.S,
            "dw": spec.dw_flops,
            "dx": 2 * spec.N * spec.P * spec.Q * spec.K * spec.C * spec.R * spec.S,
        }
        # algorithmic bytes: compress reads X and writes Z; dW reads Z and dY, writes dW
        self.bytes = {
            "compress": self.x_bytes + self.z_bytes,
            "dw": self.z_bytes + spec.N * spec.K * spec.P * spec.Q * eb + spec.K * spec.C * spec.R * spec.S * 4,
        }


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding or collectives); use --gpus 1. "
                 "The path would shard over the batch with one all-reduce of dW; see DESIGN.md.")
    import numpy as np
    import torch

    from paper_2409_11902_amd import binding as B
    from paper_2409_11902_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()  # fail loudly if the native library is missing
    if args.only == "copy":
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(args.warmup + args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"only": "copy", "bytes_read": src.numel(), "bytes_written": src.numel(),
                          "calls": args.warmup + args.steps}))
        return
    cfgs = synth.configs()
    specs = cfgs[args.workload]
    if args.layers:
        specs = [specs[int(i)] for i in args.layers.split(",")]
    t0 = time.time()
    layers = [Layer(s, args.workload, B, synth, torch) for s in specs]
    torch.cuda.synchronize()
    log(f"[bench] {args.workload}: {len(layers)} layers set up in {time.time() - t0:.1f}s")
    for L in layers:
        log(f"[bench]   {L.spec.name}: {L.plan}")

    stream = torch.cuda.current_stream()

    if args.only:
        for L in layers:
            for _ in range(args.warmup + args.steps):
                if args.only == "dw":
                    B.conv_bwd_weight_compressed(L.d, L.Z, L.dY, L.dW, L.ws[B.OP_BWD_WEIGHT_COMPRESSED], stream)
                elif args.only == "compress":
                    B.cac_compress(L.d, L.X, L.Z, stream)
                elif args.only == "fwd":
                    B.conv_fwd_and_compress(L.d, L.X, L.W, L.b, L.Y, L.Z, L.ws[B.OP_FWD_AND_COMPRESS], stream)
                else:
                    B.conv_bwd_data(L.d, L.W, L.dY, L.dX, L.ws[B.OP_BWD_DATA], stream)
        torch.cuda.synchronize()
        print(json.dumps({"only": args.only, "workload": args.workload, "calls_per_layer": args.warmup + args.steps}))
        return

    def step():
        for L in layers:
            B.conv_fwd_and_compress(L.d, L.X, L.W, L.b, L.Y, L.Z, L.ws[B.OP_FWD_AND_COMPRESS], stream)
            if args.separate_backward:
                B.conv_bwd_weight_compressed(L.d, L.Z, L.dY, L.dW, L.ws[B.OP_BWD_WEIGHT_COMPRESSED], stream)
                B.conv_bwd_data(L.d, L.W, L.dY, L.dX, L.ws[B.OP_BWD_DATA], stream)
            else:
                # both gradients of the layer in one call (same kernels and results; one launch fewer)
                B.conv_bwd_weight_and_data(L.d, L.Z, L.W, L.dY, L.dW, L.dX, L.ws[B.OP_BWD_WEIGHT_AND_DATA], stream)

    # ---- untimed warm-up (also sets kernel attributes before any capture)
    for _ in range(max(1, args.warmup)):
        step()
    torch.cuda.synchronize()

    graph = None
    if not args.no_graph:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                stream = side
                step()
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step()
            torch.cuda.synchronize()
            ref = [L.dW.clone() for L in layers]
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            assert all(torch.equal(r, L.dW) for r, L in zip(ref, layers)), "graph replay changed dW"
            graph = g
        except Exception as e:  # capture is an optimisation of the launch path only
            log(f"[bench] HIP graph capture unavailable ({type(e).__name__}: {e}); launching eagerly")
            graph = None
        stream = torch.cuda.current_stream()

    run = (lambda: graph.replay()) if graph is not None else step
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    # ---- per-op durations with events on the launch stream (instrumented loop, eager)
    nrep = max(5, min(args.steps, 30))
    names = ("fwd+compress", "dw_in_step", "dx")
    acc = {n: [0.0] * len(layers) for n in names}
    evs = []
    for _ in range(nrep):
        for i, L in enumerate(layers):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            e[0].record(stream)
            B.conv_fwd_and_compress(L.d, L.X, L.W, L.b, L.Y, L.Z, L.ws[B.OP_FWD_AND_COMPRESS], stream)
            e[1].record(stream)
            B.conv_bwd_weight_compressed(L.d, L.Z, L.dY, L.dW, L.ws[B.OP_BWD_WEIGHT_COMPRESSED], stream)
            e[2].record(stream)
            B.conv_bwd_data(L.d, L.W, L.dY, L.dX, L.ws[B.OP_BWD_DATA], stream)
            e[3].record(stream)
            evs.append((i, e))
    torch.cuda.synchronize()
    # median over the repetitions: these launches come from Python, and a repetition in which the
    # host fell behind the GPU (the interval then contains idle time) must not shift the figure
    samples = {n: [[] for _ in layers] for n in names}
    for i, e in evs:
        for j, n in enumerate(names):
            samples[n][i].append(e[j].elapsed_time(e[j + 1]))  # ms
    for n in names:
        for i in range(len(layers)):
            acc[n][i] = float(np.median(samples[n][i]))

    # ---- the weight-gradient call alone: back-to-back launches between two events on the launch stream
    dw_ms = time_dw(layers, B, torch, stream)

    # ---- compress alone: warm (same buffers) and cold (rotating through > 512 MiB)
    comp = []
    for L in layers:
        es = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for _ in range(5):
            B.cac_compress(L.d, L.X, L.Z, stream)
        es[0].record(stream)
        for _ in range(50):
            B.cac_compress(L.d, L.X, L.Z, stream)
        es[1].record(stream)
        torch.cuda.synchronize()
        warm_ms = es[0].elapsed_time(es[1]) / 50
        ncopy = max(2, int((640 << 20) // max(L.x_bytes, 1)) + 1)
        ncopy = min(ncopy, 64)
        xs = [L.X.clone() for _ in range(ncopy)]
        for x in xs:
            B.cac_compress(L.d, x, L.Z, stream)
        es = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        es[0].record(stream)
        reps = 3
        for _ in range(reps):
            for x in xs:
                B.cac_compress(L.d, x, L.Z, stream)
        es[1].record(stream)
        torch.cuda.synchronize()
        cold_ms = es[0].elapsed_time(es[1]) / (reps * ncopy)
        del xs
        comp.append((warm_ms, cold_ms))

    # ---- gradient quality (untimed): cosine of dW from the pooled map against the exact dW
    cosines = [grad_cosine(L, B, synth, torch, stream) for L in layers]

    # ---- report
    tot_flops = sum(sum(L.flops.values()) for L in layers)
    dw_flops = sum(L.flops["dw"] for L in layers)
    log(f"[bench] {'layer':28s} {'fwd+cmp us':>10s} {'dW us':>8s} {'dW TF/s':>8s} {'%peak':>6s} {'dX us':>8s} "
        f"{'cmp cold GB/s':>13s} {'%hbm':>5s} {'warm GB/s':>9s} {'X MiB':>7s} {'Z MiB':>7s} {'saved':>6s}")
    per_layer = []
    for i, L in enumerate(layers):
        dw_tf = L.flops["dw"] / (dw_ms[i] * 1e-3) / 1e12
        warm, cold = comp[i]
        cg, wg = L.bytes["compress"] / (cold * 1e-3) / 1e9, L.bytes["compress"] / (warm * 1e-3) / 1e9
        log(f"[bench] {L.spec.name:28s} {acc['fwd+compress'][i] * 1e3:10.1f} {dw_ms[i] * 1e3:8.1f} {dw_tf:8.1f} "
            f"{100 * dw_tf / PEAK_BF16_TFLOPS:6.1f} {acc['dx'][i] * 1e3:8.1f} {cg:13.0f} {100 * cg / PEAK_HBM_GBPS:5.1f} "
            f"{wg:9.0f} {L.x_bytes / 2**20:7.2f} {L.z_bytes / 2**20:7.2f} {L.x_bytes / L.z_bytes:6.2f}")
        per_layer.append({"layer": L.spec.name, "dw_us": round(dw_ms[i] * 1e3, 2), "dw_tflops": round(dw_tf, 1),
                          "dw_in_step_us": round(acc["dw_in_step"][i] * 1e3, 2),
                          "fwd_compress_us": round(acc["fwd+compress"][i] * 1e3, 2), "dx_us": round(acc["dx"][i] * 1e3, 2),
                          "compress_cold_gbps": round(cg, 1), "compress_warm_gbps": round(wg, 1),
                          "x_bytes": L.x_bytes, "z_bytes": L.z_bytes, "dw_cosine_vs_exact": round(cosines[i][0], 5),
                          "dw_cosine_vs_exact_max_pool": round(cosines[i][1], 5)})
    dw_tflops = dw_flops / (sum(dw_ms) * 1e-3) / 1e12
    comp_bytes = sum(L.bytes["compress"] for L in layers)
    comp_cold_gbps = comp_bytes / (sum(c for _, c in comp) * 1e-3) / 1e9
    x_total, z_total = sum(L.x_bytes for L in layers), sum(L.z_bytes for L in layers)
    nl = len(layers)
    traffic = read_traffic(args.workload) if not args.layers else None

    out = {
        "metric": "dW TFLOP/s + compress GB/s (% of MI355X roofline); activation bytes saved",
        "value": round(tot_flops / (ms_per_step * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s (fwd + dW-from-Z + dX algorithmic flops of one step / step time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if specs[0].dtype == synth.BF16 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "layers": [L.spec.name for L in layers], "batch": specs[0].N,
                   "pool_k": specs[0].k, "launch": "hip_graph" if graph is not None else "eager",
                   "backward": "two calls" if args.separate_backward else "conv_bwd_weight_and_data"},
        "dw_tflops": round(dw_tflops, 1), "dw_frac_of_bf16_peak": round(dw_tflops / PEAK_BF16_TFLOPS, 4),
        "compress_cold_gbps": round(comp_cold_gbps, 1), "compress_frac_of_hbm_peak": round(comp_cold_gbps / PEAK_HBM_GBPS, 4),
        "activation_bytes": {"x": x_total, "z": z_total, "saved": x_total - z_total, "ratio": round(x_total / z_total, 3)},
        # one launch = one conv_bwd_weight_compressed call on one layer = dw_mfma_kernel plus the
        # slice-sum kernel behind it; flops and duration are the means over the workload's layers
        "roofline": {"kernel": "dw_mfma_kernel + dw_reduce (the two launches of conv_bwd_weight_compressed)",
                     "bound": "mfma", "achieved": round(dw_tflops, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(dw_tflops / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                     "flops_per_launch": dw_flops // nl, "algorithmic_bytes_per_launch": sum(L.bytes["dw"] for L in layers) // nl,
                     "avg_launch_us": round(sum(dw_ms) * 1e3 / nl, 2), "launches_timed": DW_LAUNCHES},
        "roofline_compress": {"kernel": "compress_kernel (cac_compress, cold: inputs rotate through > 640 MB)",
                              "bound": "hbm", "achieved": round(comp_cold_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                              "frac": round(comp_cold_gbps / PEAK_HBM_GBPS, 4),
                              "bytes_per_launch": comp_bytes // nl,
                              "avg_launch_us": round(sum(c for _, c in comp) * 1e3 / nl, 2)},
        "per_layer": per_layer,
    }

    if args.also and args.also != args.workload and not args.layers:
        del layers
        torch.cuda.empty_cache()
        other = [Layer(s, args.also, B, synth, torch, dw_only=True) for s in cfgs[args.also]]
        oms = time_dw(other, B, torch, stream)
        out["dw_other_workloads"] = {args.also: [
            {"layer": L.spec.name, "dw_us": round(t * 1e3, 2), "dw_tflops": round(L.flops["dw"] / (t * 1e-3) / 1e12, 1),
             "frac_of_bf16_peak": round(L.flops["dw"] / (t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)} for L, t in zip(other, oms)]}
        for L, t in zip(other, oms):
            log(f"[bench] {args.also} {L.spec.name}: dW {t * 1e3:.1f} us, "
                f"{L.flops['dw'] / (t * 1e-3) / 1e12:.0f} TFLOP/s ({100 * L.flops['dw'] / (t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS:.1f}% of peak)")

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(specs, args.workload, synth, args.cpu_seconds, np)
    print(json.dumps(out), flush=True)


DW_LAUNCHES = 200


def grad_cosine(L, B, synth, torch, stream):
    """Cosine similarity (the paper's layer-sensitivity metric) between the weight gradient
    computed from the pooled map and the exact one (the same call with pooling factor 1, whose
    saved activation is X itself), all on the device.  Returns that figure for the mean (the
    paper's compression) and for the tile maximum."""
    spec1 = L.spec.with_k(1)
    d1 = B.desc_from_spec(spec1)
    n = B.cac_workspace_size(d1, B.OP_BWD_WEIGHT_COMPRESSED)
    ws1 = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda:0")
    dW1 = torch.empty_like(L.dW)
    B.conv_bwd_weight_compressed(L.d, L.Z, L.dY, L.dW, L.ws[B.OP_BWD_WEIGHT_COMPRESSED], stream)
    B.conv_bwd_weight_compressed(d1, L.X, L.dY, dW1, ws1, stream)
    out = torch.empty(4, dtype=torch.float32, device="cuda:0")
    wsc = torch.empty(B.cac_workspace_size(L.d, B.OP_GRAD_COSINE), dtype=torch.uint8, device="cuda:0")
    B.cac_grad_cosine(L.d, L.dW, dW1, out, wsc, stream)
    # the same with the tile maximum as the compression (the paper leaves other poolings open)
    dmax = B.desc_from_spec(L.spec, pool_mode=B.POOL_MAX)
    Zmax, dWmax, out2 = torch.empty_like(L.Z), torch.empty_like(L.dW), torch.empty_like(out)
    B.cac_compress(dmax, L.X, Zmax, stream)
    B.conv_bwd_weight_compressed(dmax, Zmax, L.dY, dWmax, L.ws[B.OP_BWD_WEIGHT_COMPRESSED], stream)
    B.cac_grad_cosine(L.d, dWmax, dW1, out2, wsc, stream)
    torch.cuda.synchronize()
    return float(out[0].item()), float(out2[0].item())


def time_dw(layers, B, torch, stream):
    """Mean duration (ms) of one conv_bwd_weight_compressed call per layer: 20 untimed
    launches, then DW_LAUNCHES back to back between two events recorded on the launch stream."""
    out = []
    for L in layers:
        ws = L.ws[B.OP_BWD_WEIGHT_COMPRESSED]
        for _ in range(20):
            B.conv_bwd_weight_compressed(L.d, L.Z, L.dY, L.dW, ws, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(DW_LAUNCHES):
            B.conv_bwd_weight_compressed(L.d, L.Z, L.dY, L.dW, ws, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) / DW_LAUNCHES)
    return out


def read_traffic(workload):
    """HBM bytes per conv_bwd_weight_compressed launch from the committed counter summary
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain copy of known size), or None."""
    path = os.path.join(ROOT, "profiles", f"dw_hbm_traffic_{workload}.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(float(line.split(":", 1)[1].split()[0]))
    except OSError:
        pass
    return None


def cpu_baseline(specs, config, synth, seconds, np):
    """The oracle as it stands, timed on this machine's host cores.  When a probe says
    the whole step (every layer: pooling, inflation, forward, dW from the inflated map,
    dX) fits the time budget, that is what runs; otherwise a sample of dW entries of the
    first layer at full reduction length."""
    import oracle

    def geom(sp):
        return oracle.ConvGeom(sp.N, sp.C, sp.K, sp.H, sp.W, sp.R, sp.S, sp.stride, sp.stride, sp.pad, sp.pad)

    spec = specs[0]
    host = synth.make_inputs(spec, config)
    X, dY = host["X"].astype(np.float64), host["dY"].astype(np.float64)
    Xh = oracle.inflate(oracle.avgpool(X, spec.k, spec.k), spec.H, spec.W, spec.k, spec.k)
    total = spec.K * spec.C * spec.R * spec.S
    rng = np.random.Generator(np.random.Philox(key=5))
    probe = rng.integers(0, total, 256)
    t0 = time.perf_counter()
    oracle.conv_dw_entries(geom(spec), Xh, dY, probe)
    t_probe = time.perf_counter() - t0
    flops_per_s = 2.0 * 256 * spec.N * spec.P * spec.Q / max(t_probe, 1e-9)
    if 3 * spec.dw_flops / flops_per_s <= 2.5 * seconds:
        # whole layers in order until the budget is spent (the probe's scattered entries
        # run slower than whole tensors do, so this usually covers the whole workload)
        t_total, flops, done = 0.0, 0, 0
        for sp in specs:
            if t_total > 2.5 * seconds:
                break
            done += 1
            h = synth.make_inputs(sp, config)
            X, W, b, dY = (h[k].astype(np.float64) for k in ("X", "W", "b", "dY"))
            g = geom(sp)
            t0 = time.perf_counter()
            oracle.conv_fwd(g, X, W, b)
            Xh = oracle.inflate(oracle.avgpool(X, sp.k, sp.k), sp.H, sp.W, sp.k, sp.k)
            oracle.conv_dw(g, Xh, dY)
            oracle.conv_dx(g, W, dY)
            t_total += time.perf_counter() - t0
            flops += 3 * sp.dw_flops
        return {"value": round(flops / t_total / 1e12, 5),
                "unit": "TFLOP/s (fwd + dW-from-Z + dX algorithmic flops of one step / step time)",
                "cores": oracle.num_threads(), "kind": "oracle",
                "sample": f"one step over the first {done} of {len(specs)} layers of {config} (forward, pooling, "
                          f"inflation, dW, dX of each whole layer), fp64 direct loops, {t_total:.1f}s"}
    n = int(min(total, max(256, 256 * seconds / max(t_probe, 1e-6))))
    idx = rng.integers(0, total, n)
    t0 = time.perf_counter()
    oracle.conv_dw_entries(geom(spec), Xh, dY, idx)
    t_dw = time.perf_counter() - t0
    flops = 2.0 * n * spec.N * spec.P * spec.Q
    return {"value": round(flops / t_dw / 1e12, 5), "unit": "TFLOP/s (dW entries, fp64 direct loops)",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n} of {total} dW entries of layer {spec.name} at full reduction length "
                      f"({t_dw:.1f}s; whole-layer dW extrapolates linearly to {t_dw * total / n:.0f}s)"}


if __name__ == "__main__":
    main()
