#!/usr/bin/env python3
"""Benchmark of the DS-MoE expert layer on one MI355X.

Headline (`value`): a "step" is one pass of the whole sparse-inference hot path (dsmoe_sparse_fwd: router +
softmax + selection, dispatch, grouped SwiGLU FFN, weighted combine) over one batch of synthetic tokens
already resident in HBM, on the sparse-prefill configuration "c2" (T=4096, d_model=2048, 32 experts,
d_ff=512, threshold 0.02, bf16 storage with fp32 accumulation).

Prints ONE JSON line.  `ms_per_step` / `value` come from exactly `--steps` calls bracketed by stream
synchronisation, with no instrumentation inside.  `roofline` describes the dominant kernel of the headline
workload (the grouped gate/up GEMM): algorithmic FLOPs per launch (4 * nnz * d * f) over its average duration,
measured in a separate pass with HIP events on the launch stream.  `config.summary` carries every configuration
(c2, the decode sizes c3, dense training c4, skewed prefill c5, the widened rows) in compact form: median
milliseconds of >= 20 individually timed calls, tokens/s, fraction of the relevant roofline, dominant kernel.
`config.ceilings` are micro-benchmarks run in the same process (bare MFMA loop on zero and on random operands,
cold-window streaming read and write), beside the nominal peaks.  `cpu_baseline` is the fp64 CPU checker timed
on this host.  `--verbose` adds the full per-workload records under `workloads`.
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


def csrc_digest() -> str:
    """Digest of the kernel sources: counter summaries under profiles/ name the digest they were taken with."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2404_05567_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def read_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter runs - only if they were
    taken with the kernel sources as they are now (the summary records their digest); otherwise None."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            vals[k.strip()] = v.split()[0] if v.split() else ""
    if vals.get("csrc_digest") != csrc_digest():
        return None
    try:
        return float(vals["gateup_hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def cpu_baseline(inp, cfg, passes: int):
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
    out = {"value": passes * cfg.T / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
           "sample": f"{passes} full passes of workload {cfg.name} ({cfg.T} tokens each), numpy fp64, "
                     f"{dt:.1f} s wall"}
    # context: the tiny config on one thread
    try:
        import dsmoe_inputs as gen
        from threadpoolctl import threadpool_limits
        c1 = gen.CONFIGS["c1"]
        tiny = gen.make_layer(c1, 0)
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            for _ in range(5):
                orc.sparse_forward(tiny.x, tiny.w_r, tiny.b_r, tiny.w_gate, tiny.w_up, tiny.w_down, c1.mode, c1.k, c1.eps)
            out["c1_single_thread_ms_per_pass"] = (time.perf_counter() - t0) / 5 * 1e3
    except ImportError:
        pass
    return out


class Bench:
    def __init__(self):
        import numpy as np
        import torch
        import dsmoe_inputs as gen
        import paper_2404_05567_amd as dsmoe
        self.np, self.torch, self.gen, self.dsmoe = np, torch, gen, dsmoe
        self.dev = torch.device("cuda:0")

    def to_dev(self, a, dtype):
        if a is None:
            return None
        t = self.torch.from_numpy(self.np.ascontiguousarray(a)).to(self.dev)
        return t.to(self.torch.bfloat16) if dtype == "bf16" else t

    def timed(self, fn, steps, warmup):
        """Wall-clock milliseconds per call of fn, stream-synchronised on both sides."""
        torch = self.torch
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def median_ms(self, fn, iters=20, warmup=2):
        """Median over `iters` calls, each timed by a pair of events on the stream the library launches on."""
        torch = self.torch
        for _ in range(warmup):
            fn()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        t = sorted(a.elapsed_time(b) for a, b in ev)
        return t[len(t) // 2]

    # ---- sparse prefill (c2, c5) ---------------------------------------------------------------------
    def sparse_prefill(self, name, steps, warmup, keep_inputs=False, expert="swiglu", threshold_topk=False):
        """expert="gelu": the paper's two-matrix expert on the same shapes (W_up unused, 4 nnz d f flop);
        threshold_topk: Threshold-TopK selection with the config's threshold."""
        torch, gen, dsmoe = self.torch, self.gen, self.dsmoe
        cfg = gen.CONFIGS[name]
        inp = gen.make_layer(cfg, 0)
        x, w_r, b_r = (self.to_dev(a, cfg.dtype) for a in (inp.x, inp.w_r, inp.b_r))
        w_gate, w_up, w_down = (self.to_dev(a, cfg.dtype) for a in (inp.w_gate, inp.w_up, inp.w_down))
        gelu = expert == "gelu"
        if gelu:
            w_up = None
        max_rows = cfg.T * (16 if name == "c2" else 24)
        layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=cfg.T, max_rows=max_rows, expert=expert)
        mode = dsmoe.SEL_TOPK if cfg.mode == "topk" else dsmoe.SEL_THRESHOLD
        if threshold_topk:
            mode = dsmoe.SEL_THRESHOLD_TOPK
        out = torch.empty((cfg.T, cfg.d), dtype=x.dtype, device=self.dev)

        def step():
            layer.sparse_fwd(x, w_r, b_r, w_gate, w_up, w_down, mode, cfg.k, cfg.eps, out=out)

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        assert layer.poll_error() == dsmoe.OK, "capacity overflow"
        _, _, expert_off, _ = layer.sparse_fwd_routing(cfg.T)
        eo = expert_off.cpu().numpy()
        nnz = int(eo[-1])
        ms = self.timed(step, steps, 0)                 # the timed steps: nothing but the calls
        ms_median = self.median_ms(step, max(20, min(steps, 50)))
        layer.profile_enable(steps)                     # second pass: kernel durations from events in the library
        self.timed(step, steps, 0)
        n_calls, gateup_ms, down_ms = layer.profile_read()
        layer.profile_enable(0)
        assert n_calls == steps
        assert torch.isfinite(out.float()).all()
        first_flops = (2.0 if gelu else 4.0) * nnz * cfg.d * cfg.f      # one or two products into the hidden width
        gateup_tf = first_flops / (gateup_ms / n_calls * 1e-3) / 1e12
        down_tf = 2.0 * nnz * cfg.d * cfg.f / (down_ms / n_calls * 1e-3) / 1e12
        layer_flops = first_flops + 2.0 * nnz * cfg.d * cfg.f + 2.0 * cfg.T * cfg.d * cfg.E
        res = {
            "workload": f"{name}: sparse prefill T={cfg.T} d_model={cfg.d} E={cfg.E} d_ff={cfg.f} "
                        f"{'threshold_topk' if threshold_topk else cfg.mode} eps={cfg.eps} k={cfg.k}"
                        + (" expert=gelu(x W_1) W_2" if gelu else ""),
            "tokens_per_s": cfg.T / (ms * 1e-3), "ms_per_step": ms, "median_ms": ms_median, "nnz": nnz,
            "active_fraction": nnz / (cfg.T * cfg.E),
            "rows_per_expert_min_max": [int((eo[1:] - eo[:-1]).min()), int((eo[1:] - eo[:-1]).max())],
            "layer_tflops_per_s": layer_flops / (ms * 1e-3) / 1e12,
            "layer_frac_of_bf16_peak": layer_flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "gateup_kernel_ms": gateup_ms / n_calls, "gateup_tflops_per_s": gateup_tf,
            "gateup_frac_of_bf16_peak": gateup_tf / PEAK_BF16_TFLOPS,
            "down_kernel_ms": down_ms / n_calls, "down_tflops_per_s": down_tf,
            "down_frac_of_bf16_peak": down_tf / PEAK_BF16_TFLOPS,
        }
        return (res, inp, cfg) if keep_inputs else res

    # ---- dense training forward + backward (c4) -----------------------------------------------------
    def dense_training(self, steps, warmup):
        torch, gen, dsmoe = self.torch, self.gen, self.dsmoe
        cfg = gen.CONFIGS["c4"]
        inp = gen.make_layer(cfg, 0, with_grad=True)
        w = {k: self.to_dev(getattr(inp, k), cfg.dtype) for k in ("x", "w_r", "w_gate", "w_up", "w_down", "d_out")}
        layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=cfg.T, max_rows=cfg.T)
        bufs = layer.dense_buffers(cfg.T)

        def fwd():
            layer.dense_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], buffers=bufs)

        def bwd():
            layer.dense_bwd(w["x"], w["w_r"], w["w_gate"], w["w_up"], w["w_down"], bufs["saved"], w["d_out"],
                            buffers=bufs)

        def both():
            fwd()
            bwd()

        def bwd_mi():   # total loss with the mutual-information load-balance term (Eq. 6)
            layer.dense_bwd(w["x"], w["w_r"], w["w_gate"], w["w_up"], w["w_down"], bufs["saved"], w["d_out"],
                            buffers=bufs, mi_alpha=0.01)

        def mi_loss():
            layer.mi_loss(bufs["probs"])

        ms = self.timed(both, steps, warmup)
        ms_median = self.median_ms(both, max(20, steps))
        ms_f = self.timed(fwd, steps, 1)
        ms_b = self.timed(bwd, steps, 1)
        ms_bmi = self.timed(bwd_mi, steps, 1)
        ms_mi = self.timed(mi_loss, steps, 1)
        assert torch.isfinite(bufs["dx"].float()).all()
        unit = 2.0 * cfg.T * cfg.d * cfg.E * cfg.f          # one T x d x (E f) product
        flops_f, flops_b = 3 * unit, 6 * unit
        return {
            "workload": f"c4: dense training forward+backward T={cfg.T} d_model={cfg.d} E={cfg.E} d_ff={cfg.f}",
            "tokens_per_s": cfg.T / (ms * 1e-3), "ms_per_step": ms, "median_ms": ms_median, "fwd_ms": ms_f, "bwd_ms": ms_b,
            "tflops_per_s": (flops_f + flops_b) / (ms * 1e-3) / 1e12,
            "frac_of_bf16_peak": (flops_f + flops_b) / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "fwd_frac_of_bf16_peak": flops_f / (ms_f * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "bwd_frac_of_bf16_peak": flops_b / (ms_b * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "bwd_with_mi_loss_term_ms": ms_bmi, "mi_loss_ms": ms_mi,
        }

    # ---- Mixture-of-Attention-heads forward (m2) ----------------------------------------------------
    def moa_prefill(self, steps, warmup, name="m2"):
        """The attention layer of the paper's 6B shape (Table 1) on a 2048-token prompt, every expert active
        (how the paper runs this layer at inference)."""
        torch, gen, dsmoe = self.torch, self.gen, self.dsmoe
        cfg = gen.MOA_CONFIGS[name]
        inp = gen.make_moa(cfg)
        bf = torch.bfloat16
        to = lambda a: torch.from_numpy(a).to(self.dev).to(bf)
        x, w_r, w_q, k, v, w_o = (to(a) for a in (inp.x, inp.w_r, inp.w_q, inp.k, inp.v, inp.w_o))
        layer = dsmoe.MoaLayer(cfg.d, cfg.E, cfg.n_head, cfg.d_head, max_tokens=cfg.T)
        out = torch.empty((cfg.T, cfg.d), dtype=bf, device=self.dev)
        scale = 1.0 / cfg.d_head ** 0.5
        mode = {"dense": dsmoe.SEL_ALL, "topk": dsmoe.SEL_TOPK, "threshold": dsmoe.SEL_THRESHOLD}[cfg.mode]

        def step():
            layer.fwd(x, w_r, None, w_q, k, v, w_o, mode, cfg.k, cfg.eps, scale, out=out)

        ms = self.timed(step, steps, warmup)
        ms_median = self.median_ms(step, max(20, steps))
        assert torch.isfinite(out.float()).all()
        hd = cfg.n_head * cfg.d_head
        pairs = sum(cfg.L - cfg.T + t + 1 for t in range(cfg.T))          # (query, visible key) pairs per head
        flops_proj = 2 * 2 * cfg.T * cfg.d * cfg.E * hd + 2 * cfg.T * cfg.d * cfg.E
        flops_att = 4 * cfg.E * cfg.n_head * cfg.d_head * pairs

        # dense training of the same layer: forward (every expert active) + backward
        d_out = to(gen.make_moa_upstream_grad(cfg))
        scratch = torch.empty(layer.bwd_scratch_bytes(cfg.T, cfg.L) + 256, dtype=torch.uint8, device=self.dev)
        grads = layer.bwd(x, w_r, w_q, k, v, w_o, d_out, scale, scratch=scratch) if mode == dsmoe.SEL_ALL else None
        train = {}
        if grads is not None:
            def train_step():
                layer.fwd(x, w_r, None, w_q, k, v, w_o, dsmoe.SEL_ALL, 0, 0.0, scale, out=out)
                layer.bwd(x, w_r, w_q, k, v, w_o, d_out, scale, scratch=scratch, grads=grads)

            ms_t = self.timed(train_step, steps, warmup)
            ms_t_median = self.median_ms(train_step, max(20, steps))
            assert all(torch.isfinite(g.float()).all() for g in grads.values())
            # backward: two products per projection and forward product (input and weight gradient); the attention
            # itself costs 2.5x its forward (scores again, dV, dP, dQ, dK against QK^T and PV)
            flops_bwd = 2 * (2 * 2 * cfg.T * cfg.d * cfg.E * hd) + 2.5 * flops_att + 2 * 2 * cfg.T * cfg.d * cfg.E
            train = {"train_ms_per_step": ms_t, "train_median_ms": ms_t_median, "train_tokens_per_s": cfg.T / (ms_t * 1e-3),
                     "train_tflop": (flops_proj + flops_att + flops_bwd) / 1e12,
                     "train_frac_of_bf16_peak": (flops_proj + flops_att + flops_bwd) / (ms_t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "bwd_scratch_bytes": int(scratch.numel())}
        return {
            **train,
            "workload": f"{name}: attention-expert layer forward, T={cfg.T} L={cfg.L} d_model={cfg.d} E={cfg.E} "
                        f"heads={cfg.n_head}x{cfg.d_head}, {cfg.mode}",
            "ms_per_step": ms, "median_ms": ms_median, "tokens_per_s": cfg.T / (ms * 1e-3),
            "tflop_projections": flops_proj / 1e12, "tflop_attention": flops_att / 1e12,
            "tflops_per_s": (flops_proj + flops_att) / (ms * 1e-3) / 1e12,
            "frac_of_bf16_peak": (flops_proj + flops_att) / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        }

    # ---- decode sizes (c3) --------------------------------------------------------------------------
    def decode(self, steps, warmup, n_sets=16, shape=None, tokens=(1, 8, 32, 128)):
        """T in {1, 8, 32, 128} x {top-4, threshold 0.02} on the c2 layer shape.  The loop cycles through
        `n_sets` independent weight sets (3.2 GB in all), as a model's layers would, so no call finds its
        weights in the 256 MB last-level cache.  Timed both as plain launches and as a replayed HIP graph of
        the n_sets calls (a serving loop would use the latter; it removes the host's launch cost).
        shape = (d_model, d_ff, E) runs another layer shape the same way."""
        torch, gen, dsmoe = self.torch, self.gen, self.dsmoe
        cfg = gen.CONFIGS["c3"]
        d, f, E = (cfg.d, cfg.f, cfg.E) if shape is None else shape
        router_std = cfg.router_std if shape is None else 1.5 / d ** 0.5
        g = torch.Generator(device=self.dev)
        g.manual_seed(gen.BASE_SEED + 3000)
        bf = torch.bfloat16

        def rnd(shape, std):
            return (torch.randn(shape, generator=g, device=self.dev, dtype=torch.float32) * std).to(bf)

        sets = [dict(w_r=rnd((d, E), router_std), w_gate=rnd((E, d, f), 0.02), w_up=rnd((E, d, f), 0.02),
                     w_down=rnd((E, f, d), 0.02)) for _ in range(n_sets)]
        layer = dsmoe.Layer(d, f, E, "bf16", max_tokens=128)
        results = []
        for T in tokens:
            x = rnd((T, d), 1.0)
            out = torch.empty((T, d), dtype=bf, device=self.dev)
            for mode_name, mode, k, eps in (("top4", dsmoe.SEL_TOPK, 4, 0.0), ("eps0.02", dsmoe.SEL_THRESHOLD, 0, 0.02)):
                def sweep():
                    for s in sets:
                        layer.sparse_fwd(x, s["w_r"], None, s["w_gate"], s["w_up"], s["w_down"], mode, k, eps, out=out)

                # bytes actually needed: the union of active experts per weight set
                union = []
                for s in sets:
                    layer.sparse_fwd(x, s["w_r"], None, s["w_gate"], s["w_up"], s["w_down"], mode, k, eps, out=out)
                    _, _, eo, _ = layer.sparse_fwd_routing(T)
                    eo = eo.cpu().numpy()
                    union.append(int(((eo[1:] - eo[:-1]) > 0).sum()))
                rc = layer.poll_error()
                assert rc == dsmoe.OK, f"deferred status {rc} at T={T} {mode_name}: {layer.lib.dsmoe_last_error(layer.ctx).decode()}"
                mean_union = sum(union) / len(union)
                bytes_per_call = mean_union * 3 * d * f * 2 + d * E * 2 + 2 * T * d * 2
                ms_eager = self.timed(sweep, steps, warmup) / n_sets
                ms_median = self.median_ms(sweep, max(20, steps)) / n_sets
                graph = torch.cuda.CUDAGraph()
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    sweep()
                    with torch.cuda.graph(graph, stream=side):
                        sweep()
                torch.cuda.current_stream().wait_stream(side)
                ms_graph = self.timed(graph.replay, steps, warmup) / n_sets
                best = min(ms_eager, ms_graph, ms_median)
                results.append({
                    "T": T, "selection": mode_name, "active_experts_mean": mean_union,
                    "bytes_per_call": bytes_per_call, "us_per_call_eager": ms_eager * 1e3,
                    "us_per_call_graph": ms_graph * 1e3, "us_per_call_median": ms_median * 1e3,
                    "path": DECODE_PATHS[dsmoe.sparse_fwd_path(layer, T, mode, k, eps)][0],
                    "launches": DECODE_PATHS[dsmoe.sparse_fwd_path(layer, T, mode, k, eps)][1],
                    "tokens_per_s": T / (best * 1e-3),
                    "gb_per_s": bytes_per_call / (best * 1e-3) / 1e9,
                    "frac_of_hbm_peak": bytes_per_call / (best * 1e-3) / 1e9 / PEAK_HBM_GBS,
                })
        name = "c3: sparse decode on the c2 layer" if shape is None else \
            f"sparse decode, layer d_model={d} E={E} d_ff={f}"
        return {"workload": f"{name}, {n_sets} weight sets cycled", "cases": results}


def ceilings():
    """Micro-benchmarks of this GPU, in this process: what a bare MFMA loop and a plain streaming kernel reach."""
    import torch
    import paper_2404_05567_amd as dsmoe
    out = {"nominal": {"bf16_mfma_tflops": PEAK_BF16_TFLOPS, "hbm_gb_per_s": PEAK_HBM_GBS}}
    out["mfma_bf16_zero_operands_tflops"] = max(dsmoe.bench_mfma(False, 1024, 20000) for _ in range(3))
    out["mfma_bf16_random_operands_tflops"] = max(dsmoe.bench_mfma(True, 1024, 20000) for _ in range(3))
    buf = torch.empty(3 << 30, dtype=torch.uint8, device="cuda:0")
    buf.fill_(1)
    torch.cuda.synchronize()
    med = lambda v: sorted(v)[len(v) // 2]
    out["stream_read_2GiB_gb_per_s"] = med([dsmoe.bench_stream(buf, 0, 2 << 30, False, 2048) for _ in range(5)])
    out["stream_write_2GiB_gb_per_s"] = med([dsmoe.bench_stream(buf, 0, 2 << 30, True, 2048) for _ in range(5)])
    # one decode layer's worth (200 MiB), every window cold: the buffer is walked in windows
    win = 200 << 20
    n = (3 << 30) // win
    out["stream_read_cold_200MiB_gb_per_s"] = med([dsmoe.bench_stream(buf, (i % n) * win, win, False, 1024) for i in range(2 * n)])
    out["stream_write_cold_200MiB_gb_per_s"] = med([dsmoe.bench_stream(buf, (i % n) * win, win, True, 1024) for i in range(2 * n)])
    del buf
    return out


def summarise(head, others):
    """Every configuration in a few numbers each (what the design doc's result table is made of)."""
    def prefill(r):
        return {"ms": r["ms_per_step"], "median_ms": r["median_ms"], "tokens_per_s": r["tokens_per_s"],
                "frac_bf16_peak": r["layer_frac_of_bf16_peak"], "dominant_kernel": "gateup_bf16_kernel",
                "gateup_frac": r["gateup_frac_of_bf16_peak"], "down_frac": r["down_frac_of_bf16_peak"],
                "gateup_ms": r["gateup_kernel_ms"], "down_ms": r["down_kernel_ms"], "nnz": r["nnz"]}
    out = {"c2": prefill(head)}
    for key, name in (("c3", "c3"), ("c3_largest_paper_layer", "c3_d7168_f896")):
        if key in others:
            out[name] = {f'T{c["T"]}_{c["selection"]}': {
                "us": c["us_per_call_median"], "gb_per_s": c["gb_per_s"], "frac_hbm_peak": c["frac_of_hbm_peak"],
                "active_experts": c["active_experts_mean"], "tokens_per_s": c["tokens_per_s"],
                "launches": c["launches"]} for c in others[key]["cases"]}
    if "c4" in others:
        r = others["c4"]
        out["c4"] = {"ms": r["ms_per_step"], "median_ms": r["median_ms"], "tokens_per_s": r["tokens_per_s"],
                     "frac_bf16_peak": r["frac_of_bf16_peak"], "fwd_ms": r["fwd_ms"], "bwd_ms": r["bwd_ms"],
                     "fwd_frac": r["fwd_frac_of_bf16_peak"], "bwd_frac": r["bwd_frac_of_bf16_peak"],
                     "dominant_kernel": "dense_bwd_dwgu_kernel"}
    for key in ("c5", "c2_gelu_expert", "c2_threshold_topk"):
        if key in others:
            out[key] = prefill(others[key])
    if "m2_attention_experts" in others:
        r = others["m2_attention_experts"]
        out["m2"] = {"ms": r["ms_per_step"], "median_ms": r["median_ms"], "tokens_per_s": r["tokens_per_s"],
                     "frac_bf16_peak": r["frac_of_bf16_peak"]}
        if "train_ms_per_step" in r:
            out["m2"].update({"train_fwd_bwd_ms": r["train_ms_per_step"], "train_median_ms": r["train_median_ms"],
                              "train_tokens_per_s": r["train_tokens_per_s"], "train_frac_bf16_peak": r["train_frac_of_bf16_peak"]})
    def rnd(v):
        if isinstance(v, dict):
            return {k: rnd(x) for k, x in v.items()}
        return float(f"{v:.4g}") if isinstance(v, float) else v
    return rnd(out)


# kernels dsmoe_sparse_fwd runs for a decode-sized call, by the library's own choice: description, launches
DECODE_PATHS = {
    0: ("router, dispatch, grouped GEMMs, combine", 6),
    1: ("router + weight-streaming gate/up, down, combine kernels", 4),
    2: ("one persistent kernel (all experts, router included) + partial-sum reduction", 2),
    3: ("few-token kernels: router + gate/up partial sums, activation + down partial sums, reduction", 3),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workloads", default="c2,c3,c4,c5,c2x,m2",
                    help="comma-separated subset of c2,c3,c4,c5,c2x (c2 is the headline and always runs; c2x = "
                         "c2's shapes with the GeLU two-matrix expert and with Threshold-TopK selection)")
    ap.add_argument("--cpu-passes", type=int, default=20, help="0 skips the CPU baseline")
    ap.add_argument("--decode-tokens", default="1,8,32,128", help="batch sizes of the decode workload (profiling aid)")
    ap.add_argument("--skip-large-decode", action="store_true", help="leave out the second decode layer shape")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the MFMA / streaming micro-benchmarks")
    ap.add_argument("--verbose", action="store_true", help="also print the full per-workload records (`workloads`)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run three plain device copies of this many MiB (a kernel of known HBM traffic, "
                         "used to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1")

    import torch
    import paper_2404_05567_amd as dsmoe

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dsmoe.load_library()   # no fallback: raises if the HIP library is missing
    wl = set(args.workloads.split(","))
    b = Bench()

    if args.copy_calibration > 0:
        src = torch.empty(args.copy_calibration << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head, inp, cfg = b.sparse_prefill("c2", args.steps, args.warmup, keep_inputs=True)
    side_steps = max(5, min(args.steps, 20))
    others = {}
    if "c3" in wl:
        tokens = tuple(int(v) for v in args.decode_tokens.split(","))
        others["c3"] = b.decode(side_steps, 3, tokens=tokens)
        # context: the same path on the expert layer of the largest model in the paper's speed test (Table 6:
        # embedding 7168, 32 experts of width 896), where a layer's weights are 1.2 GB and launch costs matter less
        if not args.skip_large_decode:
            others["c3_largest_paper_layer"] = b.decode(max(5, side_steps // 2), 2, n_sets=3, shape=(7168, 896, 32),
                                                        tokens=tokens)
    if "c4" in wl:
        others["c4"] = b.dense_training(side_steps, 3)
    if "c5" in wl:
        others["c5"] = b.sparse_prefill("c5", side_steps, 3)
    if "c2x" in wl:   # the rows beyond the base scope, on the headline shapes
        others["c2_gelu_expert"] = b.sparse_prefill("c2", side_steps, 3, expert="gelu")
        others["c2_threshold_topk"] = b.sparse_prefill("c2", side_steps, 3, threshold_topk=True)

    if "m2" in wl:    # the attention-expert layer (Sec. 3.2), the paper's 6B shape
        others["m2_attention_experts"] = b.moa_prefill(side_steps, 3)

    cfg_out = {"workload": "c2 (the configuration the metric is quoted on: sparse prefill, the second of the five): "
                           + head["workload"][4:],
               "nnz": head["nnz"], "active_fraction": head["active_fraction"],
               "rows_per_expert_min_max": head["rows_per_expert_min_max"], "summary": summarise(head, others)}
    if not args.no_ceilings:
        cfg_out["ceilings"] = {k: (float(f"{v:.4g}") if isinstance(v, float) else v) for k, v in ceilings().items()}
    result = {
        "metric": METRIC,
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": cfg_out,
        "roofline": {"bound": "mfma", "kernel": "gateup_bf16_kernel", "achieved": head["gateup_tflops_per_s"],
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": head["gateup_tflops_per_s"] / PEAK_BF16_TFLOPS, "traffic": read_traffic("c2")},
    }
    if args.verbose:
        result["workloads"] = others
    if args.cpu_passes > 0:
        result["cpu_baseline"] = cpu_baseline(inp, cfg, args.cpu_passes)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
