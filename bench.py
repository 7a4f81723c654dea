"""Benchmark of the MoDSE layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C4] [--mode fwd_bwd|fwd]

A step is one pass of the whole hot path over one batch of seeded synthetic input: router, permute,
grouped up-GEMM + SwiGLU, grouped down-GEMM, combine, and (mode fwd_bwd) the full backward pass.  Inputs
are resident in HBM before the timed region starts.  Prints ONE JSON line.

The default workload is C4, the training step the metric is quoted on (T = 32768, seed 1, forward +
backward).  The same line also carries, each from its own short run: `c1_fwd` (the 16K-token forward
configuration: grouped-GEMM fraction of the bf16 MFMA peak), `uniform_twin` (the equal-FLOP uniform-width layer
on the same workload, and the ratio of the two step times), `c3_fwd` (the decode-shaped configuration against
the HBM roofline).  `roofline.traffic` is measured in this run too: before this process touches the GPU it
runs itself twice under `rocprofv3 --pmc` (FETCH_SIZE, then WRITE_SIZE) on two steps of the same workload plus a
plain copy kernel of known size that calibrates the counters.
"""
from __future__ import annotations

import argparse
import csv
import glob
import json
import os
import shutil
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0    # MI355X dense bf16 MFMA peak (published)
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E peak (published)

# the launch the roofline block is about, per mode: (label, substring of its kernel name, stage it is timed as)
WGRAD_KERNEL = "gg_bf16_kernel<256, 256, 1, 4, 2, 1, 3>"
UP_KERNEL = "gg_bf16_kernel<256, 128, 2, 4, 2, 2, 0>"
CALIB_KERNEL = "CUDAFunctorOnSelf_add<float>"
CALIB_KIB = float(1 << 20)   # the calibration kernel reads 1 GiB and writes 1 GiB


def realised_flops(counts, d_ff, d):
    """Algorithmic expert FLOPs of one forward pass: 6 d sum_e n_e f_e (4 for W1/W3, 2 for W2)."""
    s = sum(int(n) * int(f) for n, f in zip(counts, d_ff))
    return 4.0 * d * s, 2.0 * d * s


def calibration_copy(torch):
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB read + 1 GiB written per launch
    b = torch.empty_like(a)
    a.fill_(1.0)
    for _ in range(3):
        torch.add(a, 1.0, out=b)   # an elementwise kernel with a recognisable name (not a DMA copy)
    torch.cuda.synchronize()
    del a, b


def _mean_kib(rows, needle):
    v = [float(r["Counter_Value"]) for r in rows if needle in r["Kernel_Name"]]
    return (sum(v) / len(v), len(v)) if v else (None, 0)


def measure_traffic(config, mode, kernel, tokens):
    """HBM bytes per launch of `kernel`: two rocprofv3 --pmc runs of this script (one counter each), each
    counter scaled by what it reads for the calibration copy.  Runs before this process touches the GPU.
    Returns (bytes or None, details)."""
    prof = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(prof):
        return None, {"note": "rocprofv3 not found"}
    out = {}
    tmp = tempfile.mkdtemp(prefix="modse_pmc_", dir=os.environ.get("TMPDIR", "/tmp"))
    try:
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            cmd = [prof, "--pmc", counter, "-d", tmp, "-o", counter.lower(), "--output-format", "csv", "--",
                   sys.executable, os.path.join(ROOT, "bench.py"), "--pmc-child", "--config", config, "--mode", mode,
                   "--tokens", str(tokens)]
            try:
                r = subprocess.run(cmd, cwd=tmp, capture_output=True, text=True, timeout=300)
            except subprocess.TimeoutExpired:
                return None, {"note": f"rocprofv3 --pmc {counter} timed out"}
            files = glob.glob(os.path.join(tmp, "**", f"{counter.lower()}*counter_collection.csv"), recursive=True)
            if r.returncode != 0 or not files:
                return None, {"note": f"rocprofv3 --pmc {counter} failed (rc {r.returncode})"}
            rows = [x for x in csv.DictReader(open(files[0])) if x["Counter_Name"] == counter]
            calib, _ = _mean_kib(rows, CALIB_KERNEL)
            kib, n = _mean_kib(rows, kernel)
            if not calib or kib is None:
                return None, {"note": f"{counter}: kernel or calibration copy not in the trace"}
            out[counter] = {"kib_per_launch": round(kib, 1), "launches": n, "calibration_kib": round(calib, 1),
                            "scale": round(CALIB_KIB / calib, 4)}
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    read = out["FETCH_SIZE"]["kib_per_launch"] * out["FETCH_SIZE"]["scale"] * 1024.0
    written = out["WRITE_SIZE"]["kib_per_launch"] * out["WRITE_SIZE"]["scale"] * 1024.0
    return read + written, {"read_bytes": round(read), "written_bytes": round(written), **out}


def cpu_baseline(cfg_name, mode, sample_tokens):
    """Times the CPU oracle, as it stands, on the first `sample_tokens` tokens of the same workload."""
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


class Run:
    """One configuration resident on the GPU: timed steps and per-stage times."""

    def __init__(self, name, mode, tokens=0):
        import workloads as wl
        from paper_2409_12210_amd.harness import LayerRunner
        cfg = wl.CONFIGS[name]
        if tokens:
            cfg = wl.with_tokens(cfg, tokens)
        bias = None
        if cfg.zipf_s is not None:
            bias = wl.load_bias_fixture(os.path.join(ROOT, "tests", "golden", f"zipf_bias_{name}.txt"))
        self.cfg, self.bwd = cfg, mode == "fwd_bwd"
        inp = wl.make_inputs(cfg, need_dy=self.bwd, logit_bias=bias)
        self.r = LayerRunner.from_inputs(inp, need_bwd=self.bwd)

    def step(self):
        self.r.fwd()
        if self.bwd:
            self.r.bwd()

    def timed(self, steps, warmup):
        import torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def timed_graph(self, steps, warmup):
        """the same step captured once into a HIP graph and replayed (what a serving loop does with a
        launch-bound step): ms per replay"""
        import torch
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            self.step()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                self.step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def stages(self, steps):
        """per-stage durations from HIP events that the library records on the launch stream"""
        import paper_2409_12210_amd as m
        m.modse_stage_timing_enable(True)
        acc = {k: 0.0 for k in m.STAGES}
        for _ in range(steps):
            self.step()
            st = m.modse_stage_times()
            for k in acc:
                acc[k] += st[k]
        m.modse_stage_timing_enable(False)
        return {k: v / steps for k, v in acc.items()}

    def flops(self):
        counts = self.r.routing_host()["counts"]
        return realised_flops(counts, self.cfg.d_ff, self.cfg.d_model), counts

    def close(self):
        import torch
        self.r = None
        torch.cuda.empty_cache()


def gemm_summary(run, st, ms_per_step):
    """TFLOP/s of the grouped-GEMM stages of one run (algorithmic FLOPs of the realised routing)."""
    (up, down), counts = run.flops()
    tf = lambda fl, ms: round(fl / (ms * 1e-3) / 1e12, 2) if ms > 0 else 0.0
    out = {"up_tflops": tf(up, st["up"]), "down_tflops": tf(down, st["down"]),
           "fwd_grouped_gemm_tflops": tf(up + down, st["up"] + st["down"])}
    out["fwd_grouped_gemm_frac_of_bf16_peak"] = round(out["fwd_grouped_gemm_tflops"] / PEAK_BF16_TFLOPS, 4)
    if run.bwd:
        out["bwd_dgrad_tflops"] = tf(up + down, st["bwd_dgrad"])
        out["bwd_wgrad_tflops"] = tf(up + down, st["bwd_wgrad"])
        gemm_ms = st["up"] + st["down"] + st["bwd_dgrad"] + st["bwd_wgrad"]
        out["all_grouped_gemm_tflops"] = tf(3 * (up + down), gemm_ms)
        out["all_grouped_gemm_frac_of_bf16_peak"] = round(out["all_grouped_gemm_tflops"] / PEAK_BF16_TFLOPS, 4)
        out["layer_tflops"] = tf(3 * (up + down), ms_per_step)
    else:
        out["layer_tflops"] = tf(up + down, ms_per_step)
    return out, counts


def hbm_stages(cfg, st, bwd):
    """HBM-bound stages: algorithmic bytes (each tensor counted once per kernel that must touch it) over stage
    time.  router: x read once (W_gate, indices and gate weights are noise); permute: indices read, x read, the k
    permuted copies written; combine: k expert-output rows read, y written."""
    b = 2 if cfg.dtype == "bf16" else 4
    T, d, k = cfg.n_tokens, cfg.d_model, cfg.top_k
    nbytes = {"route": T * d * b + 16 * T,
              "permute": T * d * b + k * T * d * b + 24 * T,
              "combine": k * T * d * b + T * d * b}
    if bwd:
        nbytes["bwd_prep"] = 3 * k * T * d * b                                     # dY rows, O -> dO, dg
        nbytes["bwd_router"] = T * d * b + k * T * d * b + T * d * b               # x, dXp rows -> dX (+ dW_gate)
    gbs = {s: round(v / (st[s] * 1e-3) / 1e9, 1) for s, v in nbytes.items() if st[s] > 0}
    names = {"route": "router"}
    return ({names.get(s, s): v for s, v in gbs.items()},
            {names.get(s, s): round(v / PEAK_HBM_GBS, 3) for s, v in gbs.items()})


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="C4")
    ap.add_argument("--mode", default="fwd_bwd", choices=["fwd_bwd", "fwd"])
    ap.add_argument("--tokens", type=int, default=0, help="override the token count of the config")
    ap.add_argument("--cpu-sample", type=int, default=32768, help="tokens for the CPU-oracle baseline (0 = skip)")
    ap.add_argument("--no-traffic", action="store_true", help="skip the two rocprofv3 --pmc runs (traffic: null)")
    ap.add_argument("--no-extras", action="store_true", help="skip the c1_fwd / uniform_twin / c3_fwd runs")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--pmc-child", action="store_true", help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the layer's hot path is single-GPU; sharding over "
              "several GPUs is a design note, not code); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import workloads as wl
    cfg0 = wl.CONFIGS[args.config]
    tokens = args.tokens or cfg0.n_tokens
    decode = tokens <= 64 and args.mode == "fwd"
    dominant = WGRAD_KERNEL if args.mode == "fwd_bwd" else UP_KERNEL

    traffic, traffic_detail = None, {"note": "not measured"}
    if not args.pmc_child and not args.no_traffic and not decode and cfg0.dtype == "bf16":
        traffic, traffic_detail = measure_traffic(args.config, args.mode, dominant, tokens)

    import torch
    import paper_2409_12210_amd as m

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    m.load_library()   # fails loudly if the HIP library is not built

    if args.pmc_child:   # the workload of the counter runs: calibration copy + two steps, nothing printed
        calibration_copy(torch)
        run = Run(args.config, args.mode, args.tokens)
        run.timed(2, 1)
        return
    if args.calib_copy:
        calibration_copy(torch)

    run = Run(args.config, args.mode, args.tokens)
    cfg = run.cfg
    T, d = cfg.n_tokens, cfg.d_model
    ms_per_step = run.timed(args.steps, args.warmup)
    st = run.stages(args.steps)
    summary, counts = gemm_summary(run, st, ms_per_step)
    near = int(run.r.routing_host()["near_tie_count"][0])
    (up_flops, down_flops), _ = run.flops()

    if decode:
        # decode-sized batch: the layer streams every expert's weights once; judged against HBM bandwidth
        wbytes = 3.0 * d * sum(cfg.d_ff) * (2 if cfg.dtype == "bf16" else 4)
        gbs = wbytes / ((st["up"] + st["down"]) * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "gg_bf16_skinny_kernel 64-row tiles (up-projection + split-K "
                                              "down-projection)",
                    "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                    "traffic": None, "bytes_per_launch": wbytes, "avg_launch_ms": round(st["up"] + st["down"], 4),
                    "whole_layer_gbs": round(wbytes / (ms_per_step * 1e-3) / 1e9, 1)}
    elif run.bwd:
        # the launch that takes the largest share of a training step: dW1, dW3 and dW2 of all experts in one grid
        fl = up_flops + down_flops   # 6 d sum_e n_e f_e: dW1 and dW3 (2 d n f each) and dW2 (2 d n f) per expert
        tfl = fl / (st["bwd_wgrad"] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "gg_bf16_kernel<EPI_STORE_F32, LAYOUT_TN>: the weight-gradient launch "
                                               "(dW1, dW3, dW2 of every expert), the longest launch of a training step",
                    "achieved": round(tfl, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tfl / PEAK_BF16_TFLOPS, 4), "traffic": traffic, "traffic_detail": traffic_detail,
                    "flops_per_launch": fl, "avg_launch_ms": round(st["bwd_wgrad"], 4)}
    else:
        tfl = up_flops / (st["up"] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "gg_bf16_kernel<EPI_SWIGLU> (grouped W1/W3 GEMM + SwiGLU), the longest "
                                               "launch of a forward pass",
                    "achieved": round(tfl, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tfl / PEAK_BF16_TFLOPS, 4), "traffic": traffic, "traffic_detail": traffic_detail,
                    "flops_per_launch": up_flops, "avg_launch_ms": round(st["up"], 4)}
    gbs, frac = hbm_stages(cfg, st, run.bwd)
    out = {
        "metric": "MoDSE layer fwd+bwd tokens/sec and grouped-GEMM % of bf16 MFMA peak (1 GPU)",
        "value": round(T / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: one MoDSE layer {args.mode}, d_model={d}, d_ff={list(cfg.d_ff)}, "
                               f"top_k={cfg.top_k}, T={T} tokens, seed {cfg.seed}",
                   "mode": args.mode, "tokens": T, "counts": [int(c) for c in counts], "near_tie_count": near},
        "stages_ms": {k: round(v, 4) for k, v in st.items()},
        "roofline": roofline,
        **summary,
        "hbm_stage_gbs": gbs, "hbm_stage_frac_of_peak": frac,
    }
    run.close()

    if not args.no_extras and args.config == "C4" and not args.tokens:
        k = max(5, args.steps // 2)
        if run.bwd:
            # the equal-FLOP layer with uniform expert widths on the same workload
            u = Run("C4U", args.mode)
            u_ms = u.timed(k, 3)
            out["uniform_twin"] = {"workload": "C4U (d_ff = 5632 x 8), same tokens and seed", "ms_per_step": round(u_ms, 4),
                                   "diverse_over_uniform": round(ms_per_step / u_ms, 4)}
            u.close()
        c1 = Run("C1", "fwd")
        c1_ms = c1.timed(k, 3)
        c1_st = c1.stages(k)
        c1_sum, _ = gemm_summary(c1, c1_st, c1_ms)
        c1_gbs, _ = hbm_stages(c1.cfg, c1_st, False)
        out["c1_fwd"] = {"workload": "C1 forward, T=16384", "ms_per_step": round(c1_ms, 4),
                         "tokens_per_s": round(16384 / (c1_ms * 1e-3), 1),
                         "stages_ms": {s: round(v, 4) for s, v in c1_st.items() if v > 0}, **c1_sum,
                         "hbm_stage_gbs": c1_gbs}
        c1.close()
        c1u = Run("C1U", "fwd")
        c1u_ms = c1u.timed(k, 3)
        out["c1_fwd"]["uniform_twin_ms"] = round(c1u_ms, 4)
        out["c1_fwd"]["diverse_over_uniform"] = round(c1_ms / c1u_ms, 4)
        c1u.close()
        c3 = Run("C3", "fwd")
        c3_ms = c3.timed(4 * k, 5)
        c3_st = c3.stages(4 * k)
        c3_graph_ms = c3.timed_graph(4 * k, 5)
        wbytes = 3.0 * c3.cfg.d_model * sum(c3.cfg.d_ff) * 2
        out["c3_fwd"] = {"workload": "C3 forward (decode-shaped), T=64", "ms_per_step": round(c3_ms, 4),
                         "ms_per_step_hip_graph": round(c3_graph_ms, 4),
                         "whole_layer_gbs_hip_graph": round(wbytes / (c3_graph_ms * 1e-3) / 1e9, 1),
                         "stages_ms": {s: round(v, 4) for s, v in c3_st.items() if v > 0},
                         "weight_bytes": wbytes,
                         "gemm_stages_gbs": round(wbytes / ((c3_st["up"] + c3_st["down"]) * 1e-3) / 1e9, 1),
                         "whole_layer_gbs": round(wbytes / (c3_ms * 1e-3) / 1e9, 1),
                         "whole_layer_frac_of_hbm_peak": round(wbytes / (c3_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        c3.close()

    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(args.config, args.mode, min(args.cpu_sample, T))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
