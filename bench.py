"""Benchmark of the MoDSE layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C1] [--mode fwd_bwd|fwd]

A step is one pass of the whole hot path over one batch of seeded synthetic input: router, permute,
grouped up-GEMM + SwiGLU, grouped down-GEMM, combine, and (mode fwd_bwd) the full backward pass.  Inputs
are resident in HBM before the timed region starts.  Prints ONE JSON line.
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

PEAK_BF16_TFLOPS = 2500.0    # MI355X dense bf16 MFMA peak (published)
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E peak (published)


def realised_flops(counts, d_ff, d):
    """Algorithmic expert FLOPs of one forward pass: 6 d sum_e n_e f_e (4 for W1/W3, 2 for W2)."""
    s = sum(int(n) * int(f) for n, f in zip(counts, d_ff))
    return 4.0 * d * s, 2.0 * d * s


def measured_traffic(cfg_name, mode):
    """HBM bytes per launch of the dominant kernel, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary
    kept under profiles/ (a line 'hbm_bytes_per_launch: N'); None if no summary covers this workload."""
    path = os.path.join(ROOT, "profiles", f"gg_bf16_swiglu_{cfg_name}_{mode}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("hbm_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(cfg_name, mode, sample_tokens):
    """Times the CPU oracle, as it stands, on the first `sample_tokens` tokens of the same workload."""
    import numpy as np
    import workloads as wl
    from oracle import modse_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    cfg = wl.with_tokens(wl.CONFIGS[cfg_name], sample_tokens)
    inp = wl.make_inputs(cfg, need_dy=True)
    t0 = time.perf_counter()
    orc.layer_fwd(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, cfg.d_ff, cfg.top_k)
    if mode == "fwd_bwd":
        orc.layer_bwd(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, cfg.d_ff, cfg.top_k, inp.dY)
    dt = time.perf_counter() - t0
    return {"value": sample_tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "seconds": round(dt, 3),
            "sample": f"first {sample_tokens} tokens of the workload, full layer {mode} in fp64 numpy"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="C1")
    ap.add_argument("--mode", default="fwd_bwd", choices=["fwd_bwd", "fwd"])
    ap.add_argument("--tokens", type=int, default=0, help="override the token count of the config")
    ap.add_argument("--cpu-sample", type=int, default=16384, help="tokens for the CPU-oracle baseline (0 = skip)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the layer's hot path is single-GPU; sharding over "
              "several GPUs is a design note, not code); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads as wl
    import paper_2409_12210_amd as m
    from paper_2409_12210_amd.harness import LayerRunner

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    m.load_library()   # fails loudly if the HIP library is not built

    cfg = wl.CONFIGS[args.config]
    if args.tokens:
        cfg = wl.with_tokens(cfg, args.tokens)
    bias = None
    if cfg.zipf_s is not None:
        bias = wl.load_bias_fixture(os.path.join(ROOT, "tests", "golden", f"zipf_bias_{args.config}.txt"))
    bwd = args.mode == "fwd_bwd"
    inp = wl.make_inputs(cfg, need_dy=bwd, logit_bias=bias)
    r = LayerRunner.from_inputs(inp, need_bwd=bwd)
    T, d = cfg.n_tokens, cfg.d_model

    def step():
        r.fwd()
        if bwd:
            r.bwd()

    if args.calib_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB read + 1 GiB written per copy
        b = torch.empty_like(a)
        a.fill_(1.0)
        for _ in range(3):
            torch.add(a, 1.0, out=b)   # an elementwise kernel with a recognisable name (not a DMA copy)
        torch.cuda.synchronize()
        del a, b

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    # per-stage durations from HIP events the library records on the launch stream
    m.modse_stage_timing_enable(True)
    acc = {k: 0.0 for k in m.STAGES}
    for _ in range(args.steps):
        step()
        st = m.modse_stage_times()
        for k in acc:
            acc[k] += st[k]
    m.modse_stage_timing_enable(False)
    stages = {k: v / args.steps for k, v in acc.items()}

    counts = r.routing_host()["counts"]
    near = int(r.routing_host()["near_tie_count"][0])
    up_flops, down_flops = realised_flops(counts, cfg.d_ff, d)
    fwd_gemm_ms = stages["up"] + stages["down"]
    fwd_gemm_tflops = (up_flops + down_flops) / (fwd_gemm_ms * 1e-3) / 1e12 if fwd_gemm_ms > 0 else 0.0
    up_tflops = up_flops / (stages["up"] * 1e-3) / 1e12 if stages["up"] > 0 else 0.0
    roofline = {"bound": "mfma", "kernel": "gg_bf16_kernel<EPI_SWIGLU> (grouped W1/W3 GEMM + SwiGLU)",
                "achieved": round(up_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(up_tflops / PEAK_BF16_TFLOPS, 4), "traffic": measured_traffic(args.config, args.mode),
                "flops_per_launch": up_flops, "avg_launch_ms": round(stages["up"], 4)}
    if T <= 64 and not bwd:
        # decode-sized batch: the layer streams every expert's weights once; judged against HBM bandwidth
        wbytes = 3.0 * d * sum(cfg.d_ff) * (2 if cfg.dtype == "bf16" else 4)
        gbs = wbytes / ((stages["up"] + stages["down"]) * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "gg_bf16_kernel 64-row tiles (up-projection + split-K down-projection)",
                    "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                    "traffic": None, "bytes_per_launch": wbytes,
                    "avg_launch_ms": round(stages["up"] + stages["down"], 4),
                    "whole_layer_gbs": round(wbytes / (ms_per_step * 1e-3) / 1e9, 1)}
    extra = {"fwd_grouped_gemm_tflops": round(fwd_gemm_tflops, 2),
             "fwd_grouped_gemm_frac_of_bf16_peak": round(fwd_gemm_tflops / PEAK_BF16_TFLOPS, 4),
             "down_gemm_tflops": round(down_flops / (stages["down"] * 1e-3) / 1e12, 2) if stages["down"] > 0 else 0}
    # HBM-bound stages: algorithmic bytes (each tensor counted once per kernel that must touch it) over stage time
    b = 2 if cfg.dtype == "bf16" else 4
    k = cfg.top_k
    hbm_bytes = {
        # router reads x; scatter reads x again and writes the k permuted copies; routing arrays are noise
        "route": T * d * b + (T * d * b + k * T * d * b) + 40 * T,
        "combine": k * T * d * b + T * d * b,
    }
    if bwd:
        hbm_bytes["bwd_prep"] = 3 * k * T * d * b                                     # dY rows, O -> dO, dg
        hbm_bytes["bwd_router"] = T * d * b + k * T * d * b + T * d * b               # x, dXp rows -> dX (+ dW_gate)
    extra["hbm_stage_gbs"] = {s: round(v / (stages[s] * 1e-3) / 1e9, 1) for s, v in hbm_bytes.items() if stages[s] > 0}
    extra["hbm_stage_frac_of_peak"] = {s: round(v / PEAK_HBM_GBS, 3) for s, v in extra["hbm_stage_gbs"].items()}
    if bwd:
        dgrad_ms, wgrad_ms = stages["bwd_dgrad"], stages["bwd_wgrad"]
        if dgrad_ms > 0:
            extra["bwd_dgrad_tflops"] = round((up_flops + down_flops) / (dgrad_ms * 1e-3) / 1e12, 2)
        if wgrad_ms > 0:
            extra["bwd_wgrad_tflops"] = round((up_flops + down_flops) / (wgrad_ms * 1e-3) / 1e12, 2)
        total_flops = 3.0 * (up_flops + down_flops)
        extra["layer_tflops"] = round(total_flops / (ms_per_step * 1e-3) / 1e12, 2)
    else:
        extra["layer_tflops"] = round((up_flops + down_flops) / (ms_per_step * 1e-3) / 1e12, 2)

    out = {
        "metric": "MoDSE layer fwd+bwd tokens/sec and grouped-GEMM % of bf16 MFMA peak (1 GPU)",
        "value": round(T / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: one MoDSE layer {args.mode}, d_model={d}, d_ff={list(cfg.d_ff)}, "
                               f"top_k={cfg.top_k}, T={T} tokens, seed {cfg.seed}",
                   "mode": args.mode, "tokens": T, "counts": [int(c) for c in counts], "near_tie_count": near},
        "stages_ms": {k: round(v, 4) for k, v in stages.items()},
        "roofline": roofline,
        **extra,
    }
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(args.config, args.mode, min(args.cpu_sample, T))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
