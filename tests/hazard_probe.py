"""Runs a fixed set of calls through whichever build of the library DSMOE_LIBRARY names and prints one JSON line
{case: sha256 of the raw output bytes}.  tests/test_gpu_conservative_waits.py runs it once per build and compares:
every sum in the library has a fixed order, so a build whose hand-counted waits are replaced by full waits must
produce the same bits.  The cases walk the shape classes of the contraction core: exact and ragged K step counts,
K tails read from the zero page, chained and plain tile loops, half tiles, K segments, every decode path."""
import hashlib
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import torch  # noqa: E402

import dsmoe_inputs as gen  # noqa: E402
import paper_2404_05567_amd as dsmoe  # noqa: E402


def digest(*tensors):
    h = hashlib.sha256()
    torch.cuda.synchronize()
    for t in tensors:
        h.update(t.detach().contiguous().cpu().view(torch.uint8).numpy().tobytes())
    return h.hexdigest()[:24]


def dev(a, bf16=True):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    return t.to(torch.bfloat16) if bf16 else t


def layer_weights(inp):
    return [dev(getattr(inp, k)) for k in ("x", "w_r", "b_r", "w_gate", "w_up", "w_down")]


def main():
    out = {}
    # sparse prefill: full and half tiles, chained (K = 512, 2048) and plain loops, both experts
    for name, T, d, E, f, expert in (("prefill_c2", 4096, 2048, 32, 512, "swiglu"), ("prefill_ragged", 777, 320, 16, 192, "swiglu"),
                                     ("prefill_gelu", 1500, 1024, 16, 256, "gelu")):
        cfg = gen.LayerConfig(name, 21, T=T, d=d, E=E, f=f, dtype="bf16", mode="threshold", k=0, eps=0.02,
                              router_std=1.5 / np.sqrt(d))
        inp = gen.make_layer(cfg, 0)
        if expert == "gelu":
            inp.w_up = None
        x, w_r, b_r, w_g, w_u, w_d = layer_weights(inp)
        layer = dsmoe.Layer(d, f, E, "bf16", max_tokens=T, expert=expert)
        o = layer.sparse_fwd(x, w_r, b_r, w_g, w_u, w_d, dsmoe.SEL_THRESHOLD, 0, 0.02)
        assert layer.poll_error() == dsmoe.OK
        out[name] = digest(o)
    # decode paths on the c3 layer
    cfg = gen.CONFIGS["c3"]
    for T in (1, 3, 8, 32, 64, 128):
        inp = gen.make_layer(cfg.with_(T=T), T)
        x, w_r, b_r, w_g, w_u, w_d = layer_weights(inp)
        layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, "bf16", max_tokens=T)
        for mode, k, eps in ((dsmoe.SEL_TOPK, 4, 0.0), (dsmoe.SEL_THRESHOLD, 0, 0.02)):
            o = layer.sparse_fwd(x, w_r, b_r, w_g, w_u, w_d, mode, k, eps)
            assert layer.poll_error() == dsmoe.OK
            out[f"decode_T{T}_path{dsmoe.sparse_fwd_path(layer, T, mode, k, eps)}_{'topk' if k else 'eps'}"] = digest(o)
    # dense training, ragged token count (K tails of the token-contracted products) and the GeLU expert
    for name, T, expert in (("dense_ragged", 777, "swiglu"), ("dense_gelu", 300, "gelu")):
        cfg = gen.LayerConfig(name, 22, T=T, d=512, E=16, f=256, dtype="bf16", mode="threshold", k=0, eps=0.02,
                              router_std=1.5 / np.sqrt(512))
        inp = gen.make_layer(cfg, 0, with_grad=True)
        if expert == "gelu":
            inp.w_up = None
        x, w_r, b_r, w_g, w_u, w_d = layer_weights(inp)
        layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, "bf16", max_tokens=T, expert=expert)
        o, _, saved = layer.dense_fwd(x, w_r, b_r, w_g, w_u, w_d, save=True)
        g = layer.dense_bwd(x, w_r, w_g, w_u, w_d, saved, dev(inp.d_out), with_bias_grad=True)
        out[name] = digest(o, *[g[k] for k in sorted(g) if g[k] is not None])
    # attention layer, forward + backward, ragged T / L
    mc = gen.MoaConfig("probe", 23, T=300, L=555, d=256, E=8, n_head=2, d_head=128, dtype="bf16", mode="dense", router_std=0.1)
    mi = gen.make_moa(mc)
    ml = dsmoe.MoaLayer(mc.d, mc.E, mc.n_head, mc.d_head, max_tokens=mc.T)
    a = [dev(v) for v in (mi.x, mi.w_r, mi.w_q, mi.k, mi.v, mi.w_o)]
    o = ml.fwd(a[0], a[1], None, a[2], a[3], a[4], a[5], dsmoe.SEL_ALL, 0, 0.0, 0.1)
    g = ml.bwd(*a, dev(gen.make_moa_upstream_grad(mc)), 0.1)
    out["moa_fwd_bwd"] = digest(o, *[g[k] for k in sorted(g)])
    print("DIGESTS " + json.dumps(out, sort_keys=True), flush=True)


if __name__ == "__main__":
    main()
