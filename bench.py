#!/usr/bin/env python3
"""Benchmark of the clustered, compressed MoE FFN layer forward on one MI355X.

A step is one pass of the whole hot path (route -> permute -> expert FFNs with shared
bases and INT4 rank-r residuals -> combine) over one batch of synthetic tokens, through
the C ABI (cmoe_forward).  Inputs and weights are resident in HBM before timing starts.

Prints ONE JSON line: whole-layer tokens/s on the named workload, a roofline object for
the dominant kernel (durations from HIP events recorded by the library on the launch
stream, in a second pass over the same steps), the same for the weight-bound
configuration, and the FP64 oracle timed on the host cores on a bounded sample.
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

PEAK_F16_TFLOPS = 2500.0     # MI355X dense FP16 matrix peak
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E peak


def kernel_work(cfg, kernel, clusters_hit, experts_hit):
    """Algorithmic flops and bytes of ONE launch of a kernel of the path (per-token
    figures of the method times the tokens a launch processes; intermediates that only
    exist because of how the path is split into kernels are not credited)."""
    T, d, f, k, r = cfg.T, cfg.d, cfg.d_ff, cfg.k, cfg.r
    if kernel == "gemm1_fused":      # W1_base x, + U1 t1, GELU, gated sum, V2 a
        flops = T * (2 * d * f + 4 * k * r * f)
        byts = clusters_hit * f * d * 2 + experts_hit * (r * f + 4 * r * f // cfg.q) + T * d * 2
    elif kernel == "gemm1_base":     # W1_base x (weight-streaming path)
        flops = T * 2 * d * f
        byts = clusters_hit * f * d * 2 + T * d * 2
    elif kernel == "residual_up":    # + U1 t1, GELU, gated sum, V2 a (weight-streaming path)
        flops = T * 4 * k * r * f
        byts = experts_hit * (r * f + 4 * r * f // cfg.q)
    elif kernel == "gemm2":          # W2_base A
        flops = T * 2 * d * f
        byts = clusters_hit * f * d * 2 + T * d * 2
    elif kernel == "t1":             # V1 x
        flops = T * 2 * k * r * d
        byts = experts_hit * (r * d // 2 + 2 * r * d // cfg.q) + T * d * 2
    elif kernel == "combine":        # + U2 s, un-permute
        flops = T * 2 * k * r * d
        byts = experts_hit * (r * d // 2 + 2 * r * d // cfg.q) + 2 * T * d * 2
    elif kernel == "route_stats":    # loads, load CV, centroid EMA (x rows read once per assignment), cluster activity
        flops = T * k * d
        byts = T * k * d * 2 + 2 * cfg.E * d * 4 + T * k * 4 + T * 4
    elif kernel == "route":
        flops = T * 2 * d * (cfg.G + cfg.K)
        byts = T * d * 2 + (cfg.G + cfg.E) * d * 2
    else:
        flops, byts = 0, 0
    return flops, byts


def run_config(cfg, steps, warmup, want_stats=False, pack=True):
    import numpy as np
    import torch

    import cmoe_inputs as ci
    import paper_2510_02345_amd as cm

    w = ci.generate(cfg)
    layer = cm.Layer(cfg.d, cfg.d_ff, cfg.G, cfg.K, cfg.r, cfg.k, cfg.q, w, cfg.T, device="cuda:0", pack=pack)
    x = torch.from_numpy(w["x"]).to("cuda:0")
    # the one-time re-tiling of the bases (done by the constructor, weights being static across
    # steps) timed on its own; it is not part of a step.  The canonical base arrays are freed
    # afterwards: every kernel reads the packed buffer, the only resident copy of the bases.
    pack_ms = 0.0
    if pack:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        layer.pack()
        torch.cuda.synchronize()
        pack_ms = (time.perf_counter() - t0) * 1e3
        layer.drop_canonical_bases()
    resident = layer.resident_weight_bytes()
    out = layer.forward_buffers(cfg.T)
    for _ in range(warmup):
        layer.forward(x, out)
    # an event after every step (on the launch stream) gives the spread next to the mean
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        layer.forward(x, out)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    ms_median = per_step[len(per_step) // 2] if steps % 2 else 0.5 * (per_step[steps // 2 - 1] + per_step[steps // 2])
    ms_min = per_step[0]

    # second pass over the same steps with per-kernel HIP events on the launch stream
    layer.timing_enable(True)
    for _ in range(steps):
        layer.forward(x, out)
    torch.cuda.synchronize()
    tm = layer.timing_read()
    layer.timing_enable(False)
    per_kernel = {n: (ms / steps) for n, (ms, cnt) in tm.items() if cnt}

    stats_ms = None
    if want_stats:
        # the routing statistics by-products on the same routing result
        E = cfg.G * cfg.K
        mu = torch.zeros((E, cfg.d), dtype=torch.float32, device="cuda:0")
        act = torch.zeros((cfg.G,), dtype=torch.float32, device="cuda:0")
        idle = torch.zeros((cfg.G,), dtype=torch.int32, device="cuda:0")
        for _ in range(3):
            layer.route_stats(x, out["perm"], out["offsets"], out["expert_idx"], mu, act, idle)
        layer.timing_enable(True)
        for _ in range(steps):
            layer.route_stats(x, out["perm"], out["offsets"], out["expert_idx"], mu, act, idle)
        torch.cuda.synchronize()
        stats_ms = layer.timing_read()["route_stats"][0] / steps
        layer.timing_enable(False)

    multi_ms = None
    if want_stats:
        # routing variant: two clusters per token, temperature, cluster-probability scaling
        om = layer.forward_multi(x, 2, 0.7, True)      # allocates the workspace and the outputs once
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(max(steps // 2, 3)):
            layer.forward_multi(x, 2, 0.7, True, out=om)
        torch.cuda.synchronize()
        multi_ms = (time.perf_counter() - t0) / max(steps // 2, 3) * 1e3
        del om

    backward_ms = None
    if want_stats:
        # backward pass for the frozen selection of this step (whole entry point between two
        # HIP events on its stream)
        dy = torch.from_numpy(np.random.default_rng(cfg.seed + 7).standard_normal((cfg.T, cfg.d)).astype(np.float16))
        dy = dy.to("cuda:0")
        grads = layer.backward(x, dy, out["expert_idx"], out["gate"])
        torch.cuda.synchronize()
        layer.timing_enable(True)
        n_bw = max(steps // 4, 3)
        for _ in range(n_bw):
            grads = layer.backward(x, dy, out["expert_idx"], out["gate"])
        torch.cuda.synchronize()
        backward_ms = layer.timing_read()["backward"][0] / n_bw
        layer.timing_enable(False)
        del grads, dy
        layer.bw_ws = None

    eidx = out["expert_idx"].cpu().numpy()
    offs = out["offsets"].cpu().numpy()
    clusters_hit = int((np.diff(offs) > 0).sum())
    experts_hit = int(len(np.unique(eidx)))
    layer.close()
    return dict(ms_per_step=ms_per_step, ms_median=ms_median, ms_min=ms_min, per_kernel_ms=per_kernel, clusters_hit=clusters_hit,
                experts_hit=experts_hit, inputs=w, stats_ms=stats_ms, multi_ms=multi_ms, backward_ms=backward_ms, pack_ms=pack_ms, resident=resident)


def roofline(cfg, res, bound, traffic_table):
    import cmoe_inputs as ci
    pk = res["per_kernel_ms"]
    dom = max(pk, key=lambda n: pk[n])
    flops, byts = kernel_work(cfg, dom, res["clusters_hit"], res["experts_hit"])
    sec = pk[dom] * 1e-3
    traffic = traffic_table.get(f"{cfg.name}:{dom}")
    if bound == "mfma":
        ach, peak, unit = flops / sec / 1e12, PEAK_F16_TFLOPS, "TFLOP/s"
    else:
        ach, peak, unit = byts / sec / 1e9, PEAK_HBM_GBS, "GB/s"
    whole_flops = ci.flops_per_token(cfg)["total"] * cfg.T
    whole_bytes = ci.algorithmic_bytes(cfg, res["clusters_hit"], res["experts_hit"])["total"]
    step_s = res["ms_per_step"] * 1e-3
    return {"bound": bound, "kernel": dom, "achieved": round(ach, 2), "peak": peak, "unit": unit,
            "frac": round(ach / peak, 4), "traffic": traffic, "kernel_ms": round(pk[dom], 4),
            "per_kernel_ms": {n: round(v, 4) for n, v in pk.items()},
            "whole_path_frac_mfma": round(whole_flops / step_s / 1e12 / PEAK_F16_TFLOPS, 4),
            "whole_path_frac_hbm": round(whole_bytes / step_s / 1e9 / PEAK_HBM_GBS, 4)}


def compress_leg(cfg, steps=3):
    """cmoe_compress on the first FFN matrix of the workload's shape: dense experts
    [E][d_ff][d] (cluster base + low-rank residual + noise, drawn on the device) -> base,
    INT4 factors, error report.  Times the whole call; the roofline figure credits the bytes
    that must move at least once (dense experts read, base and factors written)."""
    import torch

    import paper_2510_02345_amd as cm
    G, K, out_d, in_d, r, q = cfg.G, cfg.K, cfg.d_ff, cfg.d, cfg.r, cfg.q
    E = G * K
    gen = torch.Generator(device="cuda:0").manual_seed(cfg.seed)
    W = torch.empty((E, out_d, in_d), dtype=torch.float16, device="cuda:0")
    for c in range(G):
        B = torch.randn((out_d, in_d), device="cuda:0", generator=gen) / in_d ** 0.5
        for j in range(K):
            L = torch.randn((out_d, 12), device="cuda:0", generator=gen) @ torch.randn((12, in_d), device="cuda:0",
                                                                                     generator=gen)
            N = torch.randn((out_d, in_d), device="cuda:0", generator=gen)
            W[c * K + j] = (B + 0.2 * B.norm() * L / L.norm() + 0.02 * B.norm() * N / N.norm()).half()
    sketch = min(r + 8, 48)
    omega = torch.randn((sketch, in_d), device="cuda:0", generator=gen).half()
    o = cm.compress(W, omega, G, K, r, q, n_iter=2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        o = cm.compress(W, omega, G, K, r, q, n_iter=2)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    rep = o["report"].float().cpu()
    mat = E * out_d * in_d * 2
    byts = mat + G * out_d * in_d * 2 + E * r * (out_d + in_d) * (0.5 + 2.0 / q)
    # what the method as built has to move: experts read, base written, residual and its transpose
    # written, one residual stream per product (1 + 2 * n_iter + 1 = 6), experts + base read for the error
    method = mat + G * out_d * in_d * 2 + 2 * mat + 6 * mat + mat + G * out_d * in_d * 2
    gbs = byts / (ms * 1e-3) / 1e9
    return {"workload": f"W1 of {cfg.name}: {E} dense experts [{out_d}][{in_d}] f16 -> base + rank-{r} INT4 factors, "
                        f"sketch {sketch}, 2 subspace iterations",
            "ms": round(ms, 3), "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(gbs / PEAK_HBM_GBS, 4),
            "method_traffic_GBs": round(method / (ms * 1e-3) / 1e9, 1),
            "stored_error_mean": round(float(rep[:, 0].mean()), 5), "rank_r_error_mean": round(float(rep[:, 1].mean()), 5),
            "note": "achieved / frac credit only the bytes that must move once (dense experts read, base and "
                    "factors written); method_traffic_GBs counts what the randomised subspace iteration has to "
                    "move (6 streams over the FP16 residual, its construction and the error pass)"}


def cpu_baseline(cfg, w, sample):
    """The FP64 oracle (plain definition: per-expert dense FFNs) on the first `sample`
    tokens of the workload, on the host cores."""
    from oracle import cmoe_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    ws = dict(w)
    x = w["x"][:sample]
    t0 = time.perf_counter()
    orc.forward_naive(ws, x, cfg.K, cfg.k, cfg.q)
    dt = time.perf_counter() - t0
    return {"value": round(sample / dt, 2), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {sample} of {cfg.T} tokens of {cfg.name}, forward_naive (FP64, numpy/OpenBLAS), {dt:.1f} s "
                      f"of which a few seconds build the dense FP64 matrices of the experts hit, whatever the sample size"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="index into the workload list (default: largest-T)")
    ap.add_argument("--no-weight-bound", action="store_true", help="skip the weight-bound (C4) leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-compress", action="store_true", help="skip the compression-pipeline leg")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the routing-statistics and routing-variant legs (profiling runs of the layer alone)")
    ap.add_argument("--cpu-sample", type=int, default=4096)
    ap.add_argument("--no-calibration", action="store_true",
                    help="skip the matrix-core calibration leg (sustained MFMA rate with no memory traffic)")
    ap.add_argument("--no-pack", action="store_true",
                    help="read the canonical row-major bases instead of the packed copy (and dequantise the factor "
                         "panels per step above 256 tokens)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run one 256 MiB device-to-device copy (a kernel of known traffic, to scale rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import cmoe_inputs as ci
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)

    traffic_table = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic_table = json.load(open(tpath))

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cfg = ci.config(args.config)
    res = run_config(cfg, args.steps, args.warmup, want_stats=not args.no_variants, pack=not args.no_pack)
    bound = "hbm" if cfg.name == "C4" else "mfma"
    line = {
        "metric": "tokens/s through clustered-MoE FFN layer (1 GPU)",
        "value": round(cfg.T / (res["ms_per_step"] * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(res["ms_per_step"], 4),
        "ms_per_step_median": round(res["ms_median"], 4), "ms_per_step_min": round(res["ms_min"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} d_ff={cfg.d_ff} G={cfg.G} K={cfg.K} r={cfg.r} "
                               f"top_k={cfg.k} q={cfg.q} router={cfg.router}",
                   "clusters_hit": res["clusters_hit"], "experts_hit": res["experts_hit"]},
        "roofline": roofline(cfg, res, bound, traffic_table),
        "pack_weights_ms": round(res["pack_ms"], 4),
        "resident_weight_MB": round(res["resident"] / 1e6, 1),
    }
    if res["stats_ms"]:
        _, sb = kernel_work(cfg, "route_stats", res["clusters_hit"], res["experts_hit"])
        gbs = sb / (res["stats_ms"] * 1e-3) / 1e9
        line["route_stats"] = {"ms": round(res["stats_ms"], 4), "bound": "hbm", "achieved": round(gbs, 1),
                               "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                               "note": "by-product entry point (loads, load CV, centroid EMA, cluster activity); "
                                       "three launches timed together; not part of ms_per_step"}
    if res["multi_ms"]:
        line["forward_multi"] = {"ms": round(res["multi_ms"], 4), "top_g": 2, "temperature": 0.7,
                                 "scale_by_cluster_prob": True,
                                 "tokens_per_s": round(cfg.T / (res["multi_ms"] * 1e-3), 1),
                                 "vs_two_single_cluster_steps": round(res["multi_ms"] / (2 * res["ms_per_step"]), 3),
                                 "note": "cmoe_forward_multi, workspace and outputs allocated before the timed "
                                         "loop; 2 T virtual tokens through the same kernels"}
    if res["backward_ms"]:
        M = cfg.T * cfg.k
        flops = 5 * 2.0 * cfg.T * cfg.d * cfg.d_ff + 2.0 * M * cfg.r * (5 * cfg.d + 6 * cfg.d_ff)
        tf = flops / (res["backward_ms"] * 1e-3) / 1e12
        line["backward"] = {"ms": round(res["backward_ms"], 4), "bound": "mfma", "achieved": round(tf, 1),
                            "peak": PEAK_F16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_F16_TFLOPS, 4),
                            "vs_forward": round(res["backward_ms"] / res["ms_per_step"], 3),
                            "note": "cmoe_backward for the frozen selection of the step: five shared-base products "
                                    "of 2 T d d_ff flops (once per token) and eleven rank-r products per (token, "
                                    "expert) pair; all launches timed together; not part of ms_per_step"}
    if not args.no_calibration:
        import paper_2510_02345_amd as cm
        tf, ghz = cm.calibrate_mfma()
        tf0, ghz0 = cm.calibrate_mfma(zero_operands=True)
        rf = line["roofline"]
        line["mfma_sustained"] = {
            "value": round(tf, 1), "unit": "TFLOP/s", "shader_clock_GHz": round(ghz, 3),
            "frac_of_peak": round(tf / PEAK_F16_TFLOPS, 4),
            "zero_operands": {"value": round(tf0, 1), "shader_clock_GHz": round(ghz0, 3),
                              "frac_of_peak": round(tf0 / PEAK_F16_TFLOPS, 4)},
            "dominant_kernel_vs_sustained": round(rf["achieved"] / tf, 4) if rf["bound"] == "mfma" else None,
            "note": "cmoe_calibrate_mfma in this run: the grouped products' inner schedule (16 x 16 x 32 FP16 MFMAs, "
                    "fragments read from LDS, two wavefront sets) with no global traffic and every matrix-core issue "
                    "slot used on all 256 CUs. value: operands of random mantissas (what weights and activations "
                    "look like); zero_operands: the same instructions on all-zero operands. The difference is the "
                    "board's power management, which lowers the clock with the switching activity of the data; "
                    "value is the ceiling of any FP16 product on real data on this box. roofline.frac stays against "
                    "the published 2.5 PFLOP/s"}
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, res["inputs"], min(args.cpu_sample, cfg.T))
    del res
    if not args.no_weight_bound and cfg.name != "C4":
        c4 = ci.config(4)
        r4 = run_config(c4, max(args.steps, 20), max(args.warmup, 5), pack=not args.no_pack)
        line["weight_bound"] = {
            "workload": f"{c4.name}: T={c4.T} d={c4.d} d_ff={c4.d_ff} G={c4.G} K={c4.K} r={c4.r} top_k={c4.k} q={c4.q}",
            "value": round(c4.T / (r4["ms_per_step"] * 1e-3), 1), "unit": "tokens/s",
            "ms_per_step": round(r4["ms_per_step"], 4),
            "ms_per_step_median": round(r4["ms_median"], 4), "ms_per_step_min": round(r4["ms_min"], 4),
            "clusters_hit": r4["clusters_hit"], "experts_hit": r4["experts_hit"],
            "roofline": roofline(c4, r4, "hbm", traffic_table)}
    if not args.no_compress:
        line["compress"] = compress_leg(cfg)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
