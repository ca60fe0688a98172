#!/usr/bin/env python3
"""Benchmark of the compressed-activation convolution training step on one MI355X.

A step is one pass of the whole hot path over one batch of seeded synthetic
input: for every layer of the workload, conv_fwd_and_compress (forward conv +
pooling of the saved input) and conv_bwd_weight_and_data (dW from the pooled map,
dX).  Inputs are resident in HBM before the timed region.

The default run covers all five workload configurations in one process.  The
headline (`value`, `roofline`, `cpu_baseline`) is the deep small-spatial list
(3x3 512->512 on 14x14 and 7x7 maps, batch 256): the list with the most flops per
step and the one layer whose weight gradient outlasts launch overheads by far.
The other configurations are reported under `workloads`: per layer the weight
gradient against the roof that binds it, the cold compress rate, the bytes
saved, and for the ResNet-18/ImageNet list the pooling-factor sweep k = 1, 2, 4.

Prints ONE JSON line on stdout; tables go to stderr.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 vector / matrix
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E
HEADLINE = "cfg5_deep_small_spatial"
OTHERS = ("cfg1_single_fp32", "cfg2_resnet18_cifar", "cfg3_resnet50_imagenet", "cfg4_resnet18_imagenet_k1",
          "cfg4_resnet18_imagenet_k2", "cfg4_resnet18_imagenet_k4")
DW_LAUNCHES = 200           # back-to-back launches per layer behind the weight-gradient figure
COLD_BYTES = 640 << 20      # operand sets a cold measurement rotates through (above the 256 MB last-level cache)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE, help="the headline workload (value, roofline, cpu_baseline)")
    ap.add_argument("--others", default=",".join(OTHERS),
                    help="comma-separated workloads reported under `workloads` besides the headline one; '' for none")
    ap.add_argument("--layers", default="", help="comma-separated layer indices of the headline workload (default all)")
    ap.add_argument("--no-graph", action="store_true", help="launch every call from Python instead of a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-backward", action="store_true",
                    help="the step calls conv_bwd_weight_compressed and conv_bwd_data instead of conv_bwd_weight_and_data")
    ap.add_argument("--dw-algo", default="inflate", choices=["inflate", "reduced_k", "auto"],
                    help="weight-gradient kernel of the step: the one that inflates Z in LDS (default), the reduced-K form "
                         "wherever it exists, or the reduced-K form where it pays (auto)")
    ap.add_argument("--only", default="", choices=["", "dw", "dw_rk", "compress", "fwd", "dx", "copy"],
                    help="profiling aid: run just this entry point --steps times per layer (after --warmup untimed ones) "
                         "and exit (copy: a plain 256 MiB device copy, the yardstick the HBM counters are scaled by)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    return ap.parse_args()


def kernel_sources_hash():
    """Hash of the kernel sources: counter summaries under profiles/ carry the hash they were
    taken at, and a figure read from one is dropped when the sources have changed since."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2409_11902_amd", "csrc")
    for f in sorted(os.listdir(d)):
        if f.endswith((".hip", ".h")):
            h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def read_traffic(workload, layer_name=None):
    """HBM bytes per weight-gradient call from the committed counter summary (rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE, scaled by a plain copy of known size), or None when there is none or
    it was taken on other kernel sources than the ones this run uses."""
    path = os.path.join(ROOT, "profiles", f"dw_hbm_traffic_{workload}.txt")
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    stamp = [l.split(":", 1)[1].strip() for l in lines if l.startswith("kernel_sources_sha256_16:")]
    if not stamp or stamp[0] != kernel_sources_hash():
        return None
    key = f"traffic_bytes_per_launch[{layer_name}]:" if layer_name else "traffic_bytes_per_launch:"
    for l in lines:
        if l.startswith(key):
            return int(float(l.split(":", 1)[1].split()[0]))
    return None


class Layer:
    """Device buffers of one layer of a workload."""

    def __init__(self, spec, config, B, synth, torch, dw_algo=0):
        upload = B.to_device
        self.spec = spec
        self.d = B.desc_from_spec(spec, dw_algo=dw_algo)
        self.d_rk = B.desc_from_spec(spec, dw_algo=B.DW_REDUCED_K)
        self.d_auto = B.desc_from_spec(spec, dw_algo=B.DW_AUTO)
        self.has_rk = B.cac_describe_plan(self.d_rk, B.OP_BWD_WEIGHT_COMPRESSED).startswith("dw_rk")
        hp, wp, self.z_bytes, self.x_bytes = B.cac_pooled_shape(self.d)
        td = torch.float32 if spec.dtype == synth.F32 else torch.bfloat16
        dev = "cuda:0"
        self.ws = {}
        for op in (B.OP_FWD_AND_COMPRESS, B.OP_BWD_WEIGHT_COMPRESSED, B.OP_BWD_DATA, B.OP_BWD_WEIGHT_AND_DATA):
            n = max(B.cac_workspace_size(self.d, op), B.cac_workspace_size(self.d_rk, op))
            self.ws[op] = torch.empty(max(n, 16), dtype=torch.uint8, device=dev) if n else None
        self.Z = torch.empty((spec.N, spec.C, hp, wp), dtype=td, device=dev)
        self.dW = torch.empty((spec.K, spec.C, spec.R, spec.S), dtype=torch.float32, device=dev)
        t = synth.make_inputs(spec, config)
        self.X, self.W, self.b, self.dY = (upload(t[k], spec.dtype) for k in ("X", "W", "b", "dY"))
        self.Y = torch.empty((spec.N, spec.K, spec.P, spec.Q), dtype=td, device=dev)
        self.dX = torch.empty((spec.N, spec.C, spec.H, spec.W), dtype=td, device=dev)
        self.plan = B.cac_describe_plan(self.d, B.OP_BWD_WEIGHT_COMPRESSED)
        eb = spec.elem_bytes
        conv = 2 * spec.N * spec.P * spec.Q * spec.K * spec.C * spec.R * spec.S
        self.flops = {"fwd": conv, "dw": spec.dw_flops, "dx": conv}
        # algorithmic bytes: compress reads X and writes Z; dW reads Z and dY, writes dW
        self.dy_bytes = spec.N * spec.K * spec.P * spec.Q * eb
        self.bytes = {"compress": self.x_bytes + self.z_bytes,
                      "dw": self.z_bytes + self.dy_bytes + spec.K * spec.C * spec.R * spec.S * 4}
        peak = PEAK_F32_TFLOPS if spec.dtype == synth.F32 else PEAK_BF16_TFLOPS
        self.peak_tflops = peak
        # the roof that binds the weight gradient: MFMA rate or the operands' way from HBM
        self.dw_tmin_us = max(self.flops["dw"] / (peak * 1e12), self.bytes["dw"] / (PEAK_HBM_GBPS * 1e9)) * 1e6
        self.dw_bound = "mfma" if self.flops["dw"] / (peak * 1e12) >= self.bytes["dw"] / (PEAK_HBM_GBPS * 1e9) else "hbm"


def timed(torch, stream, fn, n, warm):
    """Mean duration in ms of fn() over n back-to-back calls, events on the launch stream."""
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(n):
        fn()
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def measure_workload(name, specs, args, B, synth, torch, np, detailed):
    """Sets the workload's layers up, times one step (HIP graph) and every entry point per layer."""
    t0 = time.time()
    algo = {"reduced_k": B.DW_REDUCED_K, "auto": B.DW_AUTO}.get(args.dw_algo, B.DW_INFLATE)
    layers = [Layer(s, name, B, synth, torch, dw_algo=algo) for s in specs]
    torch.cuda.synchronize()
    log(f"[bench] {name}: {len(layers)} layers set up in {time.time() - t0:.1f}s")
    stream = torch.cuda.current_stream()

    def step(st, auto=False):
        for L in layers:
            d = L.d_auto if auto else L.d
            B.conv_fwd_and_compress(d, L.X, L.W, L.b, L.Y, L.Z, L.ws[B.OP_FWD_AND_COMPRESS], st)
            if args.separate_backward:
                B.conv_bwd_weight_compressed(d, L.Z, L.dY, L.dW, L.ws[B.OP_BWD_WEIGHT_COMPRESSED], st)
                B.conv_bwd_data(d, L.W, L.dY, L.dX, L.ws[B.OP_BWD_DATA], st)
            else:
                # both gradients of the layer in one call (same kernels and results; one launch fewer)
                B.conv_bwd_weight_and_data(d, L.Z, L.W, L.dY, L.dW, L.dX, L.ws[B.OP_BWD_WEIGHT_AND_DATA], st)

    def time_step(auto):
        """ms per step (HIP graph replays where capture works) and whether a graph was used."""
        # ---- untimed warm-up (also sets kernel attributes before any capture)
        for _ in range(max(1, args.warmup if detailed else 2)):
            step(stream, auto)
        torch.cuda.synchronize()
        graph = None
        if not args.no_graph:
            try:
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    step(side, auto)
                    torch.cuda.synchronize()
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=side):
                        step(side, auto)
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
        run = (lambda: graph.replay()) if graph is not None else (lambda: step(stream, auto))
        steps, warm = (args.steps, args.warmup) if detailed else (max(5, min(args.steps, 20)), 3)
        for _ in range(warm):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3, graph is not None

    ms_per_step, graphed_step = time_step(False)
    # the same step with dw_algo = AUTO: the reduced-K weight gradient on the layers where it pays
    on_rk = [L.spec.name for L in layers if B.cac_describe_plan(L.d_auto, B.OP_BWD_WEIGHT_COMPRESSED).startswith("dw_rk")]
    ms_per_step_auto = time_step(True)[0] if (on_rk and algo == B.DW_INFLATE) else None

    rows = []
    for L in layers:
        wsd = L.ws[B.OP_BWD_WEIGHT_COMPRESSED]
        r = {"layer": L.spec.name, "k": L.spec.k}
        # the weight-gradient call alone: warm (same operands every launch)
        r["dw_ms"] = timed(torch, stream, lambda: B.conv_bwd_weight_compressed(L.d, L.Z, L.dY, L.dW, wsd, stream), DW_LAUNCHES, 20)
        # and cold: the operands rotate through more than the last-level cache holds
        nset = int(min(24, max(2, COLD_BYTES // max(L.z_bytes + L.dy_bytes, 1) + 1)))
        sets = [(L.Z, L.dY)] + [(L.Z.clone(), L.dY.clone()) for _ in range(nset - 1)]
        it = [0]

        def dw_cold():
            z, dy = sets[it[0] % nset]
            it[0] += 1
            B.conv_bwd_weight_compressed(L.d, z, dy, L.dW, wsd, stream)
        r["dw_cold_ms"] = timed(torch, stream, dw_cold, 3 * nset, nset)
        if L.has_rk:
            r["dw_rk_ms"] = timed(torch, stream, lambda: B.conv_bwd_weight_compressed(L.d_rk, L.Z, L.dY, L.dW, wsd, stream),
                                  DW_LAUNCHES, 20)
        del sets
        r["fwd_ms"] = timed(torch, stream, lambda: B.conv_fwd_and_compress(L.d, L.X, L.W, L.b, L.Y, L.Z, L.ws[B.OP_FWD_AND_COMPRESS],
                                                                        stream), 30, 5)
        r["dx_ms"] = timed(torch, stream, lambda: B.conv_bwd_data(L.d, L.W, L.dY, L.dX, L.ws[B.OP_BWD_DATA], stream), 30, 5)
        # the bias gradient (one read of dY)
        dbv = torch.empty((L.spec.K,), dtype=torch.float32, device="cuda:0")
        r["db_ms"] = timed(torch, stream, lambda: B.conv_bwd_bias(L.d, L.dY, dbv, stream), 50, 5)
        # compress alone: warm (same buffers) and cold (rotating)
        r["cmp_warm_ms"] = timed(torch, stream, lambda: B.cac_compress(L.d, L.X, L.Z, stream), 50, 5)
        ncopy = int(min(48, max(2, COLD_BYTES // max(L.x_bytes, 1) + 1)))
        xs = [L.X] + [L.X.clone() for _ in range(ncopy - 1)]
        jt = [0]

        def cmp_cold():
            B.cac_compress(L.d, xs[jt[0] % ncopy], L.Z, stream)
            jt[0] += 1
        r["cmp_cold_ms"] = timed(torch, stream, cmp_cold, 3 * ncopy, ncopy)
        # compression at the producer: normalise + activate + pool in one pass over the same rotating inputs
        Xn = torch.empty_like(L.X)
        sc = torch.full((L.spec.C,), 1.25, dtype=torch.float32, device="cuda:0")
        sh = torch.full((L.spec.C,), -0.1, dtype=torch.float32, device="cuda:0")
        kt = [0]

        def prod_cold():
            B.cac_bn_relu_fwd_compress(L.d, xs[kt[0] % ncopy], sc, sh, Xn, L.Z, None, stream)
            kt[0] += 1
        r["prod_cold_ms"] = timed(torch, stream, prod_cold, 3 * ncopy, ncopy)
        B.cac_compress(L.d, L.X, L.Z, stream)   # (Z of the layer's own input again)
        # batch normalisation's backward pass from the pooled record of its input (two launches),
        # the incoming gradient rotating through the same buffers (it has the input's shape here)
        stat = [torch.full((L.spec.C,), v, dtype=torch.float32, device="cuda:0") for v in (0.4, 1.3, 1.1)]
        dg, dbt = torch.empty_like(stat[0]), torch.empty_like(stat[0])
        bt = [0]
        nb = B.cac_workspace_size(L.d, B.OP_BN_BWD)
        wsb = torch.empty(max(nb, 16), dtype=torch.uint8, device="cuda:0")

        def bn_cold():
            B.cac_bn_bwd_compressed(L.d, L.Z, xs[bt[0] % ncopy], stat[0], stat[1], stat[2], dg, dbt, Xn, wsb, stream)
            bt[0] += 1
        r["bn_bwd_cold_ms"] = timed(torch, stream, bn_cold, 3 * ncopy, ncopy)
        del xs, Xn
        r["cos"] = grad_cosine(L, B, synth, torch, stream) if L.spec.dtype == synth.BF16 else (None, None)
        rows.append(r)

    log(f"[bench] {name}: step {ms_per_step:.3f} ms ({'hip graph' if graphed_step else 'eager'})")
    log(f"[bench] {'layer':30s} {'k':>2s} {'fwd+cmp us':>10s} {'dW us':>8s} {'cold us':>8s} {'TF/s':>7s} {'roof':>4s} {'%roof':>6s} "
        f"{'rk us':>7s} {'dX us':>8s} {'cmp cold GB/s':>13s} {'%hbm':>5s} {'X MiB':>7s} {'Z MiB':>7s} {'saved':>6s} {'cos':>6s}")
    per_layer = []
    for L, r in zip(layers, rows):
        dw_tf = L.flops["dw"] / (r["dw_ms"] * 1e-3) / 1e12
        frac_roof = L.dw_tmin_us / (r["dw_ms"] * 1e3)
        cg = L.bytes["compress"] / (r["cmp_cold_ms"] * 1e-3) / 1e9
        wg = L.bytes["compress"] / (r["cmp_warm_ms"] * 1e-3) / 1e9
        rk = r.get("dw_rk_ms")
        log(f"[bench] {L.spec.name:30s} {L.spec.k:2d} {r['fwd_ms'] * 1e3:10.1f} {r['dw_ms'] * 1e3:8.1f} {r['dw_cold_ms'] * 1e3:8.1f} "
            f"{dw_tf:7.1f} {L.dw_bound:>4s} {100 * frac_roof:6.1f} {(rk * 1e3 if rk else float('nan')):7.1f} {r['dx_ms'] * 1e3:8.1f} "
            f"{cg:13.0f} {100 * cg / PEAK_HBM_GBPS:5.1f} {L.x_bytes / 2**20:7.2f} {L.z_bytes / 2**20:7.2f} "
            f"{L.x_bytes / L.z_bytes:6.2f} {(r['cos'][0] if r['cos'][0] is not None else float('nan')):6.3f}")
        e = {"layer": L.spec.name, "k": L.spec.k, "dw_us": round(r["dw_ms"] * 1e3, 2), "dw_cold_us": round(r["dw_cold_ms"] * 1e3, 2),
             "dw_tflops": round(dw_tf, 1), "dw_flops": L.flops["dw"], "dw_bytes": L.bytes["dw"], "dw_bound": L.dw_bound,
             "dw_roof_us": round(L.dw_tmin_us, 2), "dw_frac_of_binding_roof": round(frac_roof, 4),
             "dw_frac_of_mfma_peak": round(dw_tf / L.peak_tflops, 4),
             "fwd_compress_us": round(r["fwd_ms"] * 1e3, 2), "dx_us": round(r["dx_ms"] * 1e3, 2),
             "db_us": round(r["db_ms"] * 1e3, 2), "db_gbps": round(L.dy_bytes / (r["db_ms"] * 1e-3) / 1e9, 1),
             "compress_cold_gbps": round(cg, 1), "compress_warm_gbps": round(wg, 1), "compress_bytes": L.bytes["compress"],
             "compress_cold_us": round(r["cmp_cold_ms"] * 1e3, 2),
             # normalise + activate + pool fused at the producer: reads X once, writes X' and Z
             "producer_fused_cold_us": round(r["prod_cold_ms"] * 1e3, 2),
             "producer_fused_cold_gbps": round((2 * L.x_bytes + L.z_bytes) / (r["prod_cold_ms"] * 1e-3) / 1e9, 1),
             # batch normalisation's backward pass from the pooled record: reads dY twice and Z twice, writes dX
             "bn_bwd_compressed_cold_us": round(r["bn_bwd_cold_ms"] * 1e3, 2),
             "bn_bwd_compressed_cold_gbps": round((3 * L.x_bytes + 2 * L.z_bytes) / (r["bn_bwd_cold_ms"] * 1e-3) / 1e9, 1),
             "x_bytes": L.x_bytes, "z_bytes": L.z_bytes, "saved_ratio": round(L.x_bytes / L.z_bytes, 3)}
        if rk:
            # the reduced-K form executes fewer multiply-adds for the same result: nominal flops
            # (those of the inflating form) over its time, and the executed ones against the roof
            ex = B.dw_rk_executed_flops(L.d_rk)
            e.update({"dw_reduced_k_us": round(rk * 1e3, 2), "dw_reduced_k_nominal_tflops": round(L.flops["dw"] / (rk * 1e-3) / 1e12, 1),
                      "dw_reduced_k_executed_flops": ex,
                      "dw_reduced_k_executed_frac_of_mfma_peak": round(ex / (rk * 1e-3) / 1e12 / L.peak_tflops, 4)})
        if r["cos"][0] is not None:
            e.update({"dw_cosine_vs_exact": round(r["cos"][0], 5), "dw_cosine_vs_exact_max_pool": round(r["cos"][1], 5)})
        per_layer.append(e)
    tot_flops = sum(sum(L.flops.values()) for L in layers)
    x_total, z_total = sum(L.x_bytes for L in layers), sum(L.z_bytes for L in layers)
    dw_flops = sum(L.flops["dw"] for L in layers)
    dw_ms = sum(r["dw_ms"] for r in rows)
    comp_bytes = sum(L.bytes["compress"] for L in layers)
    comp_ms = sum(r["cmp_cold_ms"] for r in rows)
    summary = {
        "workload": name, "dtype": "bf16" if specs[0].dtype == synth.BF16 else "f32", "batch": specs[0].N, "pool_k": specs[0].k,
        "ms_per_step": round(ms_per_step, 4), "step_tflops": round(tot_flops / (ms_per_step * 1e-3) / 1e12, 2),
        "launch": "hip_graph" if graphed_step else "eager",
        "dw_tflops": round(dw_flops / (dw_ms * 1e-3) / 1e12, 1),
        "dw_frac_of_binding_roof": round(sum(L.dw_tmin_us for L in layers) / (dw_ms * 1e3), 4),
        "compress_cold_gbps": round(comp_bytes / (comp_ms * 1e-3) / 1e9, 1),
        "compress_frac_of_hbm_peak": round(comp_bytes / (comp_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
        "activation_bytes": {"x": x_total, "z": z_total, "saved": x_total - z_total, "ratio": round(x_total / z_total, 3)},
        "per_layer": per_layer,
    }
    if ms_per_step_auto is not None:
        # same dW within the storage rounding of the tile sums; nominal = the definition's flops over the time
        summary["step_dw_auto"] = {"ms_per_step": round(ms_per_step_auto, 4),
                                   "step_tflops_nominal": round(tot_flops / (ms_per_step_auto * 1e-3) / 1e12, 2),
                                   "layers_on_reduced_k": on_rk}
    return summary, layers, rows, graphed_step


def measure_peaks(B, torch, stream):
    """What this box attains on a bare MFMA loop (on random numbers and on zeros: the chip's clock
    under sustained matrix load depends on the data) and on bare streams, with the library's
    yardstick kernels; launches back to back like every other figure here."""
    dev = "cuda:0"
    out = {}
    sink = torch.zeros(4096, dtype=torch.float32, device=dev)
    iters = 400
    flops = 2048 * iters * 16 * 2 * 32 * 32 * 16
    for name, src in (("random", torch.randn(16384, dtype=torch.float32, device=dev).to(torch.bfloat16)),
                      ("zeros", torch.zeros(16384, dtype=torch.bfloat16, device=dev))):
        ms = timed(torch, stream, lambda: B.cac_probe(B.PROBE_MFMA, src, sink, src.numel() * 2, iters, stream), 200, 20)
        out[f"mfma_bf16_tflops_{name}"] = round(flops / (ms * 1e-3) / 1e12, 1)
    # the same flops with 16x16x32 MFMAs, and with one wave per SIMD instead of two (random numbers)
    src = torch.randn(16384, dtype=torch.float32, device=dev).to(torch.bfloat16)
    ms = timed(torch, stream, lambda: B.cac_probe(B.PROBE_MFMA_16X16, src, sink, src.numel() * 2, iters, stream), 200, 20)
    out["mfma_bf16_tflops_random_16x16x32"] = round(flops / (ms * 1e-3) / 1e12, 1)
    ms = timed(torch, stream, lambda: B.cac_probe(B.PROBE_MFMA_1WAVE, src, sink, src.numel() * 2, iters, stream), 200, 20)
    out["mfma_bf16_tflops_random_one_wave_per_simd"] = round(flops / 2 / (ms * 1e-3) / 1e12, 1)
    n = 512 << 20
    a = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
    b = torch.empty(n, dtype=torch.uint8, device=dev)
    ms = timed(torch, stream, lambda: B.cac_probe(B.PROBE_COPY, a, b, n, 0, stream), 20, 3)
    out["hbm_copy_gbps"] = round(2 * n / (ms * 1e-3) / 1e9, 1)
    ms = timed(torch, stream, lambda: B.cac_probe(B.PROBE_READ, a, sink, n, 0, stream), 20, 3)
    out["hbm_read_gbps"] = round(n / (ms * 1e-3) / 1e9, 1)
    out["note"] = ("bare 32x32x16 bf16 MFMA loop (2048 waves, 200 launches back to back) and 512 MiB streams on this box; "
                   "data-sheet peaks: 2500 TFLOP/s, 8000 GB/s")
    log(f"[bench] measured on this box: MFMA loop {out['mfma_bf16_tflops_random']} TFLOP/s on random numbers, "
        f"{out['mfma_bf16_tflops_zeros']} on zeros; copy {out['hbm_copy_gbps']} GB/s, read {out['hbm_read_gbps']} GB/s")
    return out


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


def k_sweep(results):
    """The pooling-factor sweep on the ResNet-18/ImageNet list: per layer, the weight gradient's
    time and rate and the saved activation's bytes at k = 1 (uncompressed reference), 2 and 4."""
    by_k = {}
    for k in (1, 2, 4):
        w = results.get(f"cfg4_resnet18_imagenet_k{k}")
        if w:
            by_k[k] = {e["layer"]: e for e in w["per_layer"]}
    if 1 not in by_k or len(by_k) < 2:
        return None
    table = []
    for name, ref in by_k[1].items():
        row = {"layer": name, "x_bytes": ref["x_bytes"]}
        for k, d in sorted(by_k.items()):
            e = d[name]
            row[f"k{k}"] = {"dw_us": e["dw_us"], "dw_cold_us": e["dw_cold_us"], "dw_tflops": e["dw_tflops"], "z_bytes": e["z_bytes"],
                            "saved_ratio": e["saved_ratio"], "dw_speedup_vs_k1": round(ref["dw_us"] / e["dw_us"], 3),
                            "dw_cosine_vs_exact": e.get("dw_cosine_vs_exact")}
            if "dw_reduced_k_us" in e:
                row[f"k{k}"]["dw_reduced_k_us"] = e["dw_reduced_k_us"]
        table.append(row)
    log("[bench] pooling-factor sweep (ResNet-18/ImageNet, batch 128): dW us (saved ratio) per k")
    for row in table:
        log(f"[bench]   {row['layer']:26s} " + "  ".join(
            f"k{k}: {row[f'k{k}']['dw_us']:7.1f} us x{row[f'k{k}']['saved_ratio']:5.2f}" for k in sorted(by_k)))
    return table


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding or collectives); use --gpus 1. "
                 "The path would shard over the batch with one all-reduce of dW (K*C*R*S*4 bytes) per layer.")
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

    if args.only:
        layers = [Layer(s, args.workload, B, synth, torch) for s in specs]
        stream = torch.cuda.current_stream()
        for L in layers:
            # Z from the library's own compress pass (an MFMA on all-zero operands runs faster than on data)
            B.cac_compress(L.d, L.X, L.Z, stream)
        torch.cuda.synchronize()
        for L in layers:
            for _ in range(args.warmup + args.steps):
                if args.only == "dw":
                    B.conv_bwd_weight_compressed(L.d, L.Z, L.dY, L.dW, L.ws[B.OP_BWD_WEIGHT_COMPRESSED], stream)
                elif args.only == "dw_rk":
                    B.conv_bwd_weight_compressed(L.d_rk, L.Z, L.dY, L.dW, L.ws[B.OP_BWD_WEIGHT_COMPRESSED], stream)
                elif args.only == "compress":
                    B.cac_compress(L.d, L.X, L.Z, stream)
                elif args.only == "fwd":
                    B.conv_fwd_and_compress(L.d, L.X, L.W, L.b, L.Y, L.Z, L.ws[B.OP_FWD_AND_COMPRESS], stream)
                else:
                    B.conv_bwd_data(L.d, L.W, L.dY, L.dX, L.ws[B.OP_BWD_DATA], stream)
        torch.cuda.synchronize()
        print(json.dumps({"only": args.only, "workload": args.workload, "calls_per_layer": args.warmup + args.steps}))
        return

    peaks = measure_peaks(B, torch, torch.cuda.current_stream())
    head, layers, rows, graphed = measure_workload(args.workload, specs, args, B, synth, torch, np, detailed=True)
    for L in layers:
        log(f"[bench]   {L.spec.name}: {L.plan}")
    # the dominant kernel of the step: the weight gradient of the layer with the most flops
    i_dom = max(range(len(layers)), key=lambda i: layers[i].flops["dw"])
    Ld, rd = layers[i_dom], rows[i_dom]
    dom_tf = Ld.flops["dw"] / (rd["dw_ms"] * 1e-3) / 1e12
    i_cmp = max(range(len(layers)), key=lambda i: layers[i].bytes["compress"])
    Lc, rc = layers[i_cmp], rows[i_cmp]
    cmp_g = Lc.bytes["compress"] / (rc["cmp_cold_ms"] * 1e-3) / 1e9
    out = {
        "metric": "dW TFLOP/s + compress GB/s (% of MI355X roofline); activation bytes saved",
        "value": head["step_tflops"],
        "unit": "TFLOP/s (fwd + dW-from-Z + dX algorithmic flops of one step / step time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, "layers": [L.spec.name for L in layers], "batch": specs[0].N,
                   "pool_k": specs[0].k, "launch": "hip_graph" if graphed else "eager",
                   "backward": "two calls" if args.separate_backward else "conv_bwd_weight_and_data",
                   "dw_algo": args.dw_algo},
        "dw_tflops": head["dw_tflops"], "dw_frac_of_bf16_peak": round(head["dw_tflops"] / PEAK_BF16_TFLOPS, 4),
        "compress_cold_gbps": head["compress_cold_gbps"], "compress_frac_of_hbm_peak": head["compress_frac_of_hbm_peak"],
        "activation_bytes": head["activation_bytes"],
        # one launch = one conv_bwd_weight_compressed call on the workload's largest layer (the
        # weight-gradient kernel plus the slice-sum kernel behind it), operands warm in the last-level
        # cache as they are inside a step, where the layer's forward pass has just written them
        "roofline": {"kernel": f"conv_bwd_weight_compressed on {Ld.spec.name} (dw_mfma_kernel + dw_reduce)",
                     "bound": "mfma", "achieved": round(dom_tf, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(dom_tf / PEAK_BF16_TFLOPS, 4), "traffic": read_traffic(args.workload, Ld.spec.name),
                     "frac_of_measured_mfma_loop": round(dom_tf / peaks["mfma_bf16_tflops_random"], 4),
                     "flops_per_launch": Ld.flops["dw"], "algorithmic_bytes_per_launch": Ld.bytes["dw"],
                     "avg_launch_us": round(rd["dw_ms"] * 1e3, 2), "avg_launch_us_cold": round(rd["dw_cold_ms"] * 1e3, 2),
                     "launches_timed": DW_LAUNCHES},
        "roofline_compress": {"kernel": f"cac_compress on {Lc.spec.name} ({'compress_narrow_kernel' if Lc.spec.W in (10, 12, 14) and Lc.spec.H % 2 == 0 and Lc.spec.k == 2 else 'compress_kernel'}), cold: inputs rotate through > 640 MB",
                              "bound": "hbm", "achieved": round(cmp_g, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                              "frac": round(cmp_g / PEAK_HBM_GBPS, 4), "bytes_per_launch": Lc.bytes["compress"],
                              "frac_of_measured_read_stream": round(cmp_g / peaks["hbm_read_gbps"], 4),
                              "avg_launch_us": round(rc["cmp_cold_ms"] * 1e3, 2)},
        "measured_peaks": peaks,
        "per_layer": head["per_layer"],
    }
    if "step_dw_auto" in head:
        out["step_dw_auto"] = head["step_dw_auto"]
    del layers, rows
    torch.cuda.empty_cache()

    results = {}
    if not args.layers:
        for w in [w for w in args.others.split(",") if w and w != args.workload]:
            s, ls, _, _ = measure_workload(w, cfgs[w], args, B, synth, torch, np, detailed=False)
            results[w] = s
            del ls
            torch.cuda.empty_cache()
    if results:
        out["workloads"] = results
        sweep = k_sweep(results)
        if sweep:
            out["k_sweep_resnet18_imagenet"] = sweep
        # compress on the large tensors of the whole run (>= 49 MiB), bytes over time
        big = [e for w in list(results.values()) + [head] for e in w["per_layer"] if e["x_bytes"] >= (49 << 20)]
        if big:
            gb = sum(e["compress_bytes"] for e in big) / sum(e["compress_cold_us"] for e in big) / 1e3
            out["compress_large_tensors"] = {"tensors": len(big), "cold_gbps": round(gb, 1), "frac_of_hbm_peak": round(gb / PEAK_HBM_GBPS, 4)}
            # and on the largest single tensor of the run, with the workload it belongs to
            wl, top = max(((w, e) for w, r in list(results.items()) + [(args.workload, head)] for e in r["per_layer"]),
                          key=lambda we: we[1]["x_bytes"])
            out["roofline_compress_largest_tensor"] = {
                "kernel": f"cac_compress on {top['layer']} of {wl}, cold", "bound": "hbm",
                "achieved": top["compress_cold_gbps"], "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                "frac": round(top["compress_cold_gbps"] / PEAK_HBM_GBPS, 4), "bytes_per_launch": top["compress_bytes"],
                "avg_launch_us": top["compress_cold_us"]}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(specs, args.workload, synth, args.cpu_seconds, np)
    print(json.dumps(out), flush=True)


def cpu_baseline(specs, config, synth, seconds, np):
    """The oracle as it stands, timed on this machine's host cores, in the unit of `value`.  When a
    probe says the whole step (every layer: pooling, inflation, forward, dW from the inflated map,
    dX) fits the time budget, that is what runs; otherwise seeded samples of the outputs of the
    workload's largest layer, each a full-length sum: Y elements, dW entries and dX elements in
    equal shares of flops (the whole step extrapolates linearly: every output is independent)."""
    import oracle

    def geom(sp):
        return oracle.ConvGeom(sp.N, sp.C, sp.K, sp.H, sp.W, sp.R, sp.S, sp.stride, sp.stride, sp.pad, sp.pad)

    unit = "TFLOP/s (fwd + dW-from-Z + dX algorithmic flops of one step / step time)"
    spec = max(specs, key=lambda s: s.dw_flops)
    host = synth.make_inputs(spec, config)
    X, W, b, dY = (host[k].astype(np.float64) for k in ("X", "W", "b", "dY"))
    g = geom(spec)
    t0 = time.perf_counter()
    Xh = oracle.inflate(oracle.avgpool(X, spec.k, spec.k), spec.H, spec.W, spec.k, spec.k)
    t_pool = time.perf_counter() - t0
    total = spec.K * spec.C * spec.R * spec.S
    rng = np.random.Generator(np.random.Philox(key=5))
    probe = rng.integers(0, total, 256)
    t0 = time.perf_counter()
    oracle.conv_dw_entries(g, Xh, dY, probe)
    t_probe = time.perf_counter() - t0
    flops_per_s = 2.0 * 256 * spec.N * spec.P * spec.Q / max(t_probe, 1e-9)
    step_flops = sum(3 * s.dw_flops for s in specs)
    if step_flops / flops_per_s <= 2.5 * seconds:
        t_total, flops, done = 0.0, 0, 0
        for sp in specs:
            if t_total > 2.5 * seconds:
                break
            done += 1
            h = synth.make_inputs(sp, config)
            X, W, b, dY = (h[k].astype(np.float64) for k in ("X", "W", "b", "dY"))
            gg = geom(sp)
            t0 = time.perf_counter()
            oracle.conv_fwd(gg, X, W, b)
            Xh = oracle.inflate(oracle.avgpool(X, sp.k, sp.k), sp.H, sp.W, sp.k, sp.k)
            oracle.conv_dw(gg, Xh, dY)
            oracle.conv_dx(gg, W, dY)
            t_total += time.perf_counter() - t0
            flops += 3 * sp.dw_flops
        return {"value": round(flops / t_total / 1e12, 5), "unit": unit, "cores": oracle.num_threads(), "kind": "oracle",
                "sample": f"one step over the first {done} of {len(specs)} layers of {config} (forward, pooling, "
                          f"inflation, dW, dX of each whole layer), fp64 direct loops, {t_total:.1f}s"}
    # sampled outputs: a third of the time budget each, every count sized by a probe of its own
    per_dw = 2.0 * spec.N * spec.P * spec.Q
    per_y = 2.0 * spec.C * spec.R * spec.S
    n_all_y, n_all_x = spec.N * spec.K * spec.P * spec.Q, spec.N * spec.C * spec.H * spec.W

    def sized(fn, n_probe, n_all):
        t0 = time.perf_counter()
        fn(n_probe)
        per_entry = (time.perf_counter() - t0) / n_probe
        return int(min(n_all, max(n_probe, seconds / 3 / max(per_entry, 1e-12))))

    n_dw = sized(lambda n: oracle.conv_dw_entries(g, Xh, dY, rng.integers(0, total, n)), 4096, total)
    n_y = sized(lambda n: oracle.conv_fwd_entries(g, X, W, b, rng.integers(0, n_all_y, n)), 65536, n_all_y)
    n_x = sized(lambda n: oracle.conv_dx_entries(g, W, dY, rng.integers(0, n_all_x, n)), 65536, n_all_x)
    t0 = time.perf_counter()
    oracle.conv_dw_entries(g, Xh, dY, rng.integers(0, total, n_dw))
    t_dw = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.conv_fwd_entries(g, X, W, b, rng.integers(0, spec.N * spec.K * spec.P * spec.Q, n_y))
    t_y = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.conv_dx_entries(g, W, dY, rng.integers(0, spec.N * spec.C * spec.H * spec.W, n_x))
    t_x = time.perf_counter() - t0
    # a dX element sums over the taps that reach it: on average R*S/stride^2 per output channel
    per_x = 2.0 * spec.K * spec.R * spec.S / (spec.stride ** 2)
    flops = n_dw * per_dw + n_y * per_y + n_x * per_x
    t_all = t_dw + t_y + t_x
    return {"value": round(flops / t_all / 1e12, 5), "unit": unit, "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"layer {spec.name} of {config}: {n_dw} of {total} dW entries ({t_dw:.1f}s), {n_y} Y elements ({t_y:.1f}s), "
                      f"{n_x} dX elements ({t_x:.1f}s), each at full reduction length, fp64 direct loops; pooling + inflation of "
                      f"the whole layer took {t_pool:.1f}s (not in the rate); the whole step ({step_flops / 1e9:.0f} GFLOP) "
                      f"extrapolates linearly to {step_flops / (flops / t_all):.0f}s"}


if __name__ == "__main__":
    main()
