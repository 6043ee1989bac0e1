"""GPU parity of the dense-training forward and backward (Sec. 3.2 "Dense Training", Eq. 3) against the
CPU checker, through the C ABI.

Bar: every output tensor (O, the scores, and each gradient separately) within
max|gpu - ref| / max|ref| <= 1e-5 (fp32) or 2e-2 (bf16 storage, fp32 accumulation).
"""
import sys

import numpy as np
import pytest

import dsmoe_inputs as gen
from oracle import dsmoe_oracle as orc
from tests import helpers

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available()
    return torch


@pytest.fixture(scope="module")
def dsmoe():
    import paper_2404_05567_amd as m
    m.load_library()      # raises if the HIP library is missing: there is no fallback
    return m


def dev(torch, a, dtype):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_dev(torch, inp):
    dt = inp.cfg.dtype
    return {k: dev(torch, getattr(inp, k), dt) for k in ("x", "w_r", "b_r", "w_gate", "w_up", "w_down", "d_out")}


def host(t):
    return t.float().cpu().numpy()


def check_dense(torch, dsmoe, cfg, bias=False, variant=0):
    T, E, tol = cfg.T, cfg.E, TOL[cfg.dtype]
    say(f"[case] dense {cfg.name} T={T} d={cfg.d} E={E} f={cfg.f} {cfg.dtype} bias={bias}")
    inp = gen.make_layer(cfg, variant, with_grad=True)
    if bias and inp.b_r is None:
        g = np.random.default_rng(cfg.index)
        inp.b_r = gen.round_to_bf16(g.standard_normal(E).astype(np.float32) * 0.5) if cfg.dtype == "bf16" \
            else (g.standard_normal(E) * 0.5).astype(np.float32)
    w = to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, E, cfg.dtype, max_tokens=max(T, 1))

    O_ref, S_ref, _ = orc.dense_forward(inp.x, inp.w_r, inp.b_r, inp.w_gate, inp.w_up, inp.w_down)
    gr = orc.dense_backward(inp.x, inp.w_r, inp.b_r, inp.w_gate, inp.w_up, inp.w_down, inp.d_out)

    out, probs, saved = layer.dense_fwd(w["x"], w["w_r"], w["b_r"], w["w_gate"], w["w_up"], w["w_down"],
                                        want_probs=True, save=True)
    torch.cuda.synchronize()
    assert helpers.rel_err(host(probs), S_ref) <= 1e-5
    err = helpers.rel_err(host(out), O_ref)
    say(f"  forward rel err {err:.3e}")
    assert err <= tol

    # inference-only forward (nothing saved) gives the same output
    out2, _, _ = layer.dense_fwd(w["x"], w["w_r"], w["b_r"], w["w_gate"], w["w_up"], w["w_down"])
    torch.cuda.synchronize()
    assert torch.equal(out, out2)

    g = layer.dense_bwd(w["x"], w["w_r"], w["w_gate"], w["w_up"], w["w_down"], saved, w["d_out"],
                        with_bias_grad=bias)
    torch.cuda.synchronize()
    refs = dict(dx=gr.dX, dw_r=gr.dW_r, dw_gate=gr.dW_gate, dw_up=gr.dW_up, dw_down=gr.dW_down)
    if bias:
        refs["db_r"] = gr.db_r
    for name, ref in refs.items():
        e = helpers.rel_err(host(g[name]), ref)
        say(f"  {name} rel err {e:.3e}")
        assert e <= tol, name
    return layer, w, saved, g


def test_c1_dense_forward_and_backward_fp32(torch, dsmoe):
    check_dense(torch, dsmoe, gen.CONFIGS["c1"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_shapes_with_router_bias(torch, dsmoe, dtype):
    # T below / not a multiple of any tile or K step, ragged column tiles, several tiles per expert
    for T, d, E, f in [(77, 192, 8, 64), (333, 320, 16, 192)]:
        cfg = gen.LayerConfig("dense_ragged", 21, T=T, d=d, E=E, f=f, dtype=dtype, mode="topk", k=1,
                              router_std=0.08)
        check_dense(torch, dsmoe, cfg, bias=True)


def test_bf16_multi_tile(torch, dsmoe):
    cfg = gen.LayerConfig("dense_mid", 22, T=1000, d=512, E=8, f=512, dtype="bf16", mode="topk", k=1,
                          router_std=1.5 / np.sqrt(512))
    check_dense(torch, dsmoe, cfg)


def test_sixty_four_experts(torch, dsmoe):
    cfg = gen.LayerConfig("dense_e64", 23, T=200, d=256, E=64, f=64, dtype="bf16", mode="topk", k=1,
                          router_std=0.1)
    check_dense(torch, dsmoe, cfg, bias=True)


def test_repeated_backward_is_bitwise_identical(torch, dsmoe):
    cfg = gen.LayerConfig("dense_det", 24, T=600, d=256, E=8, f=128, dtype="bf16", mode="topk", k=1,
                          router_std=0.1)
    layer, w, saved, g1 = check_dense(torch, dsmoe, cfg)
    g2 = layer.dense_bwd(w["x"], w["w_r"], w["w_gate"], w["w_up"], w["w_down"], saved, w["d_out"])
    torch.cuda.synchronize()
    for k in ("dx", "dw_r", "dw_gate", "dw_up", "dw_down"):
        assert torch.equal(g1[k], g2[k]), k


def test_no_tokens(torch, dsmoe):
    cfg = gen.CONFIGS["c1"]
    inp = gen.make_layer(cfg.with_(T=0), 0, with_grad=True)
    w = to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=8)
    out, _, saved = layer.dense_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], save=True)
    assert out.shape[0] == 0
    g = layer.dense_bwd(w["x"], w["w_r"], w["w_gate"], w["w_up"], w["w_down"], saved, w["d_out"], with_bias_grad=True)
    torch.cuda.synchronize()
    for k in ("dw_r", "db_r", "dw_gate", "dw_up", "dw_down"):
        assert float(g[k].abs().max().item()) == 0.0


def test_forward_without_saved_needs_room_in_the_workspace(torch, dsmoe):
    cfg = gen.CONFIGS["c1"]
    inp = gen.make_layer(cfg, 0)
    w = to_dev(torch, gen.make_layer(cfg, 0, with_grad=True))
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=cfg.T, max_rows=cfg.T * 2)
    with pytest.raises(dsmoe.DsmoeError) as ei:
        layer.dense_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"])
    assert ei.value.code == dsmoe.ERR_WORKSPACE
    out, _, _ = layer.dense_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], save=True)
    torch.cuda.synchronize()
    O_ref, _, _ = orc.dense_forward(inp.x, inp.w_r, None, inp.w_gate, inp.w_up, inp.w_down)
    assert helpers.rel_err(host(out), O_ref) <= 1e-5


# --------------------------------------------------------------------------------------------------
# full training size, in the launch configuration bench.py times
# --------------------------------------------------------------------------------------------------
def test_c4_full_size_dense_training(torch, dsmoe):
    cfg = gen.CONFIGS["c4"]
    T, E, tol = cfg.T, cfg.E, TOL["bf16"]
    say("[case] full-size c4: generating inputs")
    inp = gen.make_layer(cfg, 0, with_grad=True)
    w = to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, E, cfg.dtype, max_tokens=T, max_rows=T)
    out, probs, saved = layer.dense_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"],
                                        want_probs=True, save=True)
    g = layer.dense_bwd(w["x"], w["w_r"], w["w_gate"], w["w_up"], w["w_down"], saved, w["d_out"])
    torch.cuda.synchronize()
    say("[case] full-size c4: GPU done, checker running")

    # every output element against the checker: all tokens of O and dX, the router gradient, and the weight
    # gradients of all experts, a slab of tokens at a time (the checker keeps e_j(X) for the slab: Eq. 3 literally)
    S_ref = orc.route(inp.x, inp.w_r, None)
    assert helpers.rel_err(host(probs), S_ref) <= 1e-5
    O_ref = np.zeros((T, cfg.d))
    dX_ref = np.zeros((T, cfg.d))
    dW_r = np.zeros((cfg.d, E))
    dWg, dWu, dWd = (np.zeros(a.shape) for a in (inp.w_gate, inp.w_up, inp.w_down))
    w_r64 = inp.w_r.astype(np.float64)
    for lo in range(0, T, 1024):
        tok = np.arange(lo, min(T, lo + 1024))
        O_ref[tok], _, Y = orc.dense_forward(inp.x, inp.w_r, None, inp.w_gate, inp.w_up, inp.w_down, tokens=tok)
        dZ = orc.softmax_backward(S_ref[tok], orc.grad_scores(Y, inp.d_out[tok]))
        del Y
        dW_r += inp.x[tok].astype(np.float64).T @ dZ
        dX_ref[tok] = dZ @ w_r64.T
        for j in range(E):
            dx_j, g_j, u_j, d_j = orc.expert_backward(inp.x[tok], S_ref[tok, j], inp.w_gate[j], inp.w_up[j],
                                                      inp.w_down[j], inp.d_out[tok])
            dX_ref[tok] += dx_j
            dWg[j] += g_j
            dWu[j] += u_j
            dWd[j] += d_j
        say(f"  checker: tokens {lo}..{tok[-1]} done")
    for name, got, ref in (("out", out, O_ref), ("dx", g["dx"], dX_ref), ("dw_r", g["dw_r"], dW_r),
                           ("dw_gate", g["dw_gate"], dWg), ("dw_up", g["dw_up"], dWu), ("dw_down", g["dw_down"], dWd)):
        e = helpers.rel_err(host(got), ref)
        say(f"  {name} (every element) rel err {e:.3e}")
        assert e <= tol, name
    for k in ("dx", "dw_r", "dw_gate", "dw_up", "dw_down"):
        assert bool(torch.isfinite(g[k].float()).all()), k


# --------------------------------------------------------------------------------------------------
# mutual-information load-balance loss (Sec. 3.2, Eq. 4-6) and its gradient through the router
# --------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("T,E", [(1, 8), (128, 8), (777, 32), (8192, 32), (5000, 64)])
def test_mi_loss_matches_the_checker(torch, dsmoe, T, E):
    say(f"[case] mi_loss T={T} E={E}")
    g = np.random.default_rng(100 + T + E)
    Z = g.standard_normal((T, E)) * 1.5
    S = orc.softmax_rows(Z).astype(np.float32)
    layer = dsmoe.Layer(64, 64, E, "f32", max_tokens=T)
    loss, p_mean = layer.mi_loss(torch.from_numpy(S).to("cuda:0"))
    torch.cuda.synchronize()
    ref = orc.mi_loss(S)
    got = float(loss.cpu()[0])
    say(f"  loss {got:.7f} ref {ref:.7f}")
    assert abs(got - ref) <= 1e-5 * max(1.0, abs(ref))
    np.testing.assert_allclose(p_mean.cpu().numpy(), S.astype(np.float64).mean(axis=0), rtol=1e-5)


def test_mi_loss_closed_forms_on_the_gpu(torch, dsmoe):
    E, T = 8, 64
    layer = dsmoe.Layer(64, 64, E, "f32", max_tokens=T)
    uniform = torch.full((T, E), 1.0 / E, dtype=torch.float32, device="cuda:0")
    onehot = torch.zeros((T, E), dtype=torch.float32, device="cuda:0")
    onehot[torch.arange(T), torch.arange(T) % E] = 1.0       # balanced one-hot: exercises 0 log 0 = 0
    collapsed = torch.zeros((T, E), dtype=torch.float32, device="cuda:0")
    collapsed[:, 3] = 1.0
    for S, want in ((uniform, 0.0), (onehot, -np.log(E)), (collapsed, 0.0)):
        loss, _ = layer.mi_loss(S)
        torch.cuda.synchronize()
        assert abs(float(loss.cpu()[0]) - want) <= 1e-6, (float(loss.cpu()[0]), want)


@pytest.mark.parametrize("name,T", [("c1", 128), ("c4", 300)])
def test_dense_backward_with_the_mi_loss_term(torch, dsmoe, name, T):
    """Total loss L_LM + alpha L_MI (Eq. 6): dx, dW_r and db_r gain the load-balance term, the expert-weight
    gradients do not change."""
    base = gen.CONFIGS[name]
    cfg = base if name == "c1" else base.with_(name="c4_small", T=T, d=512, f=128, router_std=1.5 / np.sqrt(512))
    tol = TOL[cfg.dtype]
    inp = gen.make_layer(cfg, 3, with_grad=True)
    w = to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=cfg.T)
    gr = orc.dense_backward(inp.x, inp.w_r, inp.b_r, inp.w_gate, inp.w_up, inp.w_down, inp.d_out)
    # the weight of the term is chosen so that it matters in the router gradient (half of the largest entry of
    # the language-model part), or the test would check nothing; the gradient is linear in alpha
    unit = orc.mi_backward(inp.x, inp.w_r, inp.b_r, 1.0)[1]
    alpha = float(np.float32(0.5 * np.abs(gr.dW_r).max() / np.abs(unit).max()))
    say(f"[case] dense backward + MI term {cfg.name} T={cfg.T} alpha={alpha:.4g}")
    mdx, mdw, mdb = orc.mi_backward(inp.x, inp.w_r, inp.b_r, alpha)

    _, _, saved = layer.dense_fwd(w["x"], w["w_r"], w["b_r"], w["w_gate"], w["w_up"], w["w_down"], save=True)
    g = layer.dense_bwd(w["x"], w["w_r"], w["w_gate"], w["w_up"], w["w_down"], saved, w["d_out"],
                        with_bias_grad=True, mi_alpha=alpha)
    torch.cuda.synchronize()
    for key, ref in (("dx", gr.dX + mdx), ("dw_r", gr.dW_r + mdw), ("db_r", gr.db_r + mdb),
                     ("dw_gate", gr.dW_gate), ("dw_up", gr.dW_up), ("dw_down", gr.dW_down)):
        err = helpers.rel_err(host(g[key]), ref)
        say(f"  {key} rel err {err:.3e}")
        assert err <= tol, key
    # alpha = 0 is the plain backward
    g0 = layer.dense_bwd(w["x"], w["w_r"], w["w_gate"], w["w_up"], w["w_down"], saved, w["d_out"], with_bias_grad=True)
    torch.cuda.synchronize()
    assert helpers.rel_err(host(g0["dw_r"]), gr.dW_r) <= tol


# --------------------------------------------------------------------------------------------------
# the paper's two-matrix GeLU expert (Sec. 4.1) in dense training
# --------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,T,bias", [("c1", 128, False), ("c1", 100, True), ("c4", 300, False), ("c4", 777, True)])
def test_dense_training_with_the_gelu_expert(torch, dsmoe, name, T, bias):
    base = gen.CONFIGS[name]
    cfg = base.with_(name=f"{name}_gelu", T=T) if name == "c1" else \
        base.with_(name="c4_small_gelu", T=T, d=512, f=128 if T == 300 else 192, router_std=1.5 / np.sqrt(512))
    tol = TOL[cfg.dtype]
    say(f"[case] dense GeLU expert {cfg.name} T={cfg.T} d={cfg.d} E={cfg.E} f={cfg.f} {cfg.dtype} bias={bias}")
    inp = gen.make_layer(cfg, 5, with_grad=True)
    inp.w_up = None
    if bias:
        g = np.random.default_rng(cfg.index + 50)
        b = (g.standard_normal(cfg.E) * 0.5).astype(np.float32)
        inp.b_r = gen.round_to_bf16(b) if cfg.dtype == "bf16" else b
    w = to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=cfg.T, expert="gelu")
    O_ref, S_ref, _ = orc.dense_forward(inp.x, inp.w_r, inp.b_r, inp.w_gate, None, inp.w_down)
    gr = orc.dense_backward(inp.x, inp.w_r, inp.b_r, inp.w_gate, None, inp.w_down, inp.d_out)

    out, probs, saved = layer.dense_fwd(w["x"], w["w_r"], w["b_r"], w["w_gate"], None, w["w_down"],
                                        want_probs=True, save=True)
    torch.cuda.synchronize()
    assert helpers.rel_err(host(probs), S_ref) <= 1e-5
    err = helpers.rel_err(host(out), O_ref)
    say(f"  forward rel err {err:.3e}")
    assert err <= tol
    out2, _, _ = layer.dense_fwd(w["x"], w["w_r"], w["b_r"], w["w_gate"], None, w["w_down"])   # nothing saved
    torch.cuda.synchronize()
    assert torch.equal(out2, out)

    g = layer.dense_bwd(w["x"], w["w_r"], w["w_gate"], None, w["w_down"], saved, w["d_out"], with_bias_grad=True)
    torch.cuda.synchronize()
    assert g["dw_up"] is None
    for key, ref in (("dx", gr.dX), ("dw_r", gr.dW_r), ("db_r", gr.db_r), ("dw_gate", gr.dW_gate),
                     ("dw_down", gr.dW_down)):
        err = helpers.rel_err(host(g[key]), ref)
        say(f"  {key} rel err {err:.3e}")
        assert err <= tol, key
