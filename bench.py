#!/usr/bin/env python3
"""Benchmark of the DS-MoE expert layer on one MI355X.

A "step" is one pass of the whole sparse-inference hot path (dsmoe_sparse_fwd: router + softmax +
selection, dispatch, grouped SwiGLU FFN, weighted combine) over one batch of synthetic tokens that is
already resident in HBM.  The default workload is the sparse-prefill configuration ("c2": T=4096,
d_model=2048, 32 experts, d_ff=512, threshold 0.02, bf16 storage with fp32 accumulation).

Prints ONE JSON line.  `roofline` describes the dominant kernel (the grouped gate/up GEMM): algorithmic
FLOPs per launch (4 * nnz * d * f) over its average duration, measured with HIP events on the launch
stream during the timed steps.  `cpu_baseline` is the fp64 CPU checker timed on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0
METRIC = "MoE-layer tokens/s + % bf16 MFMA peak (prefill) / % HBM BW (decode)"


def read_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from committed rocprofv3 counter runs, if any."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            try:
                vals[k.strip()] = float(v.split()[0])
            except ValueError:
                pass
    return vals.get("gateup_hbm_bytes_per_launch")


def cpu_baseline(inp, cfg, passes: int):
    import numpy as np
    from oracle import dsmoe_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    t0 = time.perf_counter()
    for _ in range(passes):
        orc.sparse_forward(inp.x, inp.w_r, inp.b_r, inp.w_gate, inp.w_up, inp.w_down, cfg.mode, cfg.k, cfg.eps)
    dt = time.perf_counter() - t0
    return {"value": passes * cfg.T / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{passes} full passes of workload {cfg.name} ({cfg.T} tokens each), numpy fp64, "
                      f"{dt:.1f} s wall"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c2", choices=["c2", "c5"])
    ap.add_argument("--cpu-passes", type=int, default=20, help="0 skips the CPU baseline")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    import dsmoe_inputs as gen
    import paper_2404_05567_amd as dsmoe

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dsmoe.load_library()   # no fallback: raises if the HIP library is missing

    cfg = gen.CONFIGS[args.config]
    inp = gen.make_layer(cfg, 0)
    dev = torch.device("cuda:0")

    def to_dev(a):
        if a is None:
            return None
        t = torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        return t.to(torch.bfloat16) if cfg.dtype == "bf16" else t

    x, w_r, b_r = to_dev(inp.x), to_dev(inp.w_r), to_dev(inp.b_r)
    w_gate, w_up, w_down = to_dev(inp.w_gate), to_dev(inp.w_up), to_dev(inp.w_down)
    max_rows = cfg.T * (16 if cfg.name == "c2" else 24)
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=cfg.T, max_rows=max_rows)
    mode = dsmoe.SEL_TOPK if cfg.mode == "topk" else dsmoe.SEL_THRESHOLD
    out = torch.empty((cfg.T, cfg.d), dtype=x.dtype, device=dev)

    def step():
        layer.sparse_fwd(x, w_r, b_r, w_gate, w_up, w_down, mode, cfg.k, cfg.eps, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert layer.poll_error() == dsmoe.OK, "capacity overflow"
    _, _, expert_off, _ = layer.sparse_fwd_routing(cfg.T)
    nnz = int(expert_off[-1].item())

    layer.profile_enable(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    n_calls, gateup_ms, down_ms = layer.profile_read()
    layer.profile_enable(0)
    assert n_calls == args.steps
    assert torch.isfinite(out.float()).all()

    ms_per_step = dt / args.steps * 1e3
    gateup_flops = 4.0 * nnz * cfg.d * cfg.f
    gateup_avg_s = gateup_ms / n_calls * 1e-3
    achieved = gateup_flops / gateup_avg_s / 1e12
    layer_flops = 6.0 * nnz * cfg.d * cfg.f + 2.0 * cfg.T * cfg.d * cfg.E
    result = {
        "metric": METRIC,
        "value": cfg.T / (dt / args.steps),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: sparse prefill T={cfg.T} d_model={cfg.d} E={cfg.E} d_ff={cfg.f} "
                               f"{cfg.mode} eps={cfg.eps} k={cfg.k}",
                   "nnz": nnz, "active_fraction": nnz / (cfg.T * cfg.E),
                   "layer_tflops_per_s": layer_flops / (dt / args.steps) / 1e12,
                   "layer_frac_of_bf16_peak": layer_flops / (dt / args.steps) / 1e12 / PEAK_BF16_TFLOPS,
                   "down_kernel_ms": down_ms / n_calls, "gateup_kernel_ms": gateup_ms / n_calls},
        "roofline": {"bound": "mfma", "kernel": "gateup_kernel", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": read_traffic(cfg.name)},
    }
    if args.cpu_passes > 0:
        result["cpu_baseline"] = cpu_baseline(inp, cfg, args.cpu_passes)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
