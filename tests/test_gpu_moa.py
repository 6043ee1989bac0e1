"""GPU parity of the Mixture-of-Attention-heads forward (Sec. 3.2, Eq. 7-8) against the checker, through the C ABI."""
import sys

import numpy as np
import pytest

import dsmoe_inputs as gen
from oracle import dsmoe_oracle as orc
from oracle import moa_oracle as moa
from tests import helpers

pytestmark = pytest.mark.gpu
TOL = 2e-2     # bf16 storage, fp32 accumulation: max |err| / max |ref|


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch as t
    if not t.cuda.is_available():
        pytest.skip("no GPU")
    return t


@pytest.fixture(scope="module")
def dsmoe():
    import paper_2404_05567_amd as m
    m.load_library()
    return m


def dev(torch, a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0").to(torch.bfloat16)


def run_and_check(torch, dsmoe, inp, mode, k=0, eps=0.0, scale=None):
    cfg = inp.cfg
    scale = 1.0 / np.sqrt(cfg.d_head) if scale is None else scale
    say(f"[case] moa {cfg.name} T={cfg.T} L={cfg.L} d={cfg.d} E={cfg.E} heads={cfg.n_head}x{cfg.d_head} mode={mode} "
        f"k={k} eps={eps} scale={scale:.4f}")
    layer = dsmoe.MoaLayer(cfg.d, cfg.E, cfg.n_head, cfg.d_head, max_tokens=max(cfg.T, 1))
    code = {"dense": dsmoe.SEL_ALL, "topk": dsmoe.SEL_TOPK, "threshold": dsmoe.SEL_THRESHOLD}[mode]
    out = layer.fwd(dev(torch, inp.x), dev(torch, inp.w_r), dev(torch, inp.b_r), dev(torch, inp.w_q), dev(torch, inp.k),
                    dev(torch, inp.v), dev(torch, inp.w_o), code, k, eps, float(scale))
    probs, mask = layer.routing(cfg.T)
    torch.cuda.synchronize()
    O_ref, S_ref, M_ref = moa.moa_forward(inp.x, inp.w_r, inp.b_r, inp.w_q, inp.k, inp.v, inp.w_o, mode, k, eps, scale)
    S_gpu = probs.cpu().numpy()
    assert helpers.rel_err(S_gpu, S_ref) <= 1e-5
    m = mask.cpu().numpy().astype(np.uint64)
    M_gpu = ((m[:, None] >> np.arange(cfg.E, dtype=np.uint64)[None, :]) & np.uint64(1)).astype(bool)
    # the selection is bit-exact: same sets as the checker's decision on the GPU's own fp32 scores and (margin-
    # conditioned inputs) as its fp64 decision
    M_same = np.ones_like(M_ref) if mode == "dense" else orc.select(S_gpu, mode, k, np.float32(eps))
    np.testing.assert_array_equal(M_gpu, M_same)
    np.testing.assert_array_equal(M_gpu, M_ref)
    err = helpers.rel_err(out.float().cpu().numpy(), O_ref)
    say(f"  rel err {err:.3e}")
    assert err <= TOL
    return out


def conditioned(cfg, variant=0):
    inp = gen.make_moa(cfg, variant)
    if cfg.mode != "dense":
        helpers.condition_margins(inp, cfg.mode, cfg.k, cfg.eps)
    return inp


@pytest.mark.parametrize("mode,k,eps", [("topk", 2, 0.0), ("threshold", 0, 0.1), ("dense", 0, 0.0)])
def test_m1_tiny(torch, dsmoe, mode, k, eps):
    cfg = gen.MOA_CONFIGS["m1"].with_(mode=mode, k=k, eps=eps)
    run_and_check(torch, dsmoe, conditioned(cfg), mode, k, eps)


def test_the_printed_formula_has_no_scale(torch, dsmoe):
    cfg = gen.MOA_CONFIGS["m1"]
    run_and_check(torch, dsmoe, conditioned(cfg), "topk", 2, 0.0, scale=1.0)


@pytest.mark.parametrize("T,L,n_head,d_head", [(300, 300, 4, 128), (130, 517, 2, 128), (1, 200, 2, 64), (257, 290, 2, 64)])
def test_ragged_tiles_and_cache_offsets(torch, dsmoe, T, L, n_head, d_head):
    cfg = gen.MoaConfig("ragged", 13, T=T, L=L, d=256, E=8, n_head=n_head, d_head=d_head, dtype="bf16", mode="topk",
                        k=3, router_std=0.08)
    run_and_check(torch, dsmoe, conditioned(cfg), "topk", 3, 0.0)


def test_sixteen_experts_of_the_1b_shape(torch, dsmoe):
    # DS-MoE-1B row of Table 1 at a reduced width: 16 experts of 2 heads of 64
    cfg = gen.MoaConfig("e16", 14, T=200, L=200, d=512, E=16, n_head=2, d_head=64, dtype="bf16", mode="threshold",
                        eps=0.05, router_std=0.06)
    run_and_check(torch, dsmoe, conditioned(cfg), "threshold", 0, 0.05)


def test_sixty_four_experts_of_one_head(torch, dsmoe):
    cfg = gen.MoaConfig("e64", 15, T=100, L=1100, d=256, E=64, n_head=1, d_head=64, dtype="bf16", mode="topk", k=5,
                        router_std=0.1)
    run_and_check(torch, dsmoe, conditioned(cfg), "topk", 5, 0.0)


def test_repeated_calls_are_bitwise_identical_and_no_tokens(torch, dsmoe):
    cfg = gen.MOA_CONFIGS["m1"]
    inp = conditioned(cfg)
    a = run_and_check(torch, dsmoe, inp, "topk", 2, 0.0)
    b = run_and_check(torch, dsmoe, inp, "topk", 2, 0.0)
    assert torch.equal(a, b)
    layer = dsmoe.MoaLayer(cfg.d, cfg.E, cfg.n_head, cfg.d_head, max_tokens=8)
    empty = torch.empty((0, cfg.d), dtype=torch.bfloat16, device="cuda:0")
    out = layer.fwd(empty, dev(torch, inp.w_r), None, dev(torch, inp.w_q), dev(torch, inp.k), dev(torch, inp.v),
                    dev(torch, inp.w_o), dsmoe.SEL_ALL)
    assert out.shape == (0, cfg.d)


def test_m2_full_size_prefill_sampled(torch, dsmoe):
    """The 6B shape of Table 1 at 2048 tokens, every expert active; the checker computes a sample of the tokens
    one by one (a token's output depends on the cache and its own row only)."""
    cfg = gen.MOA_CONFIGS["m2"]
    inp = gen.make_moa(cfg)
    scale = 1.0 / np.sqrt(cfg.d_head)
    say(f"[case] moa m2 full size T={cfg.T} L={cfg.L}")
    layer = dsmoe.MoaLayer(cfg.d, cfg.E, cfg.n_head, cfg.d_head, max_tokens=cfg.T)
    out = layer.fwd(dev(torch, inp.x), dev(torch, inp.w_r), None, dev(torch, inp.w_q), dev(torch, inp.k), dev(torch, inp.v),
                    dev(torch, inp.w_o), dsmoe.SEL_ALL, 0, 0.0, float(scale))
    torch.cuda.synchronize()
    o = out.float().cpu().numpy()
    assert np.isfinite(o).all()
    rng = np.random.default_rng(3)
    sample = np.unique(np.concatenate([[0, 1, 127, 128, cfg.T - 1], rng.integers(0, cfg.T, size=64)]))
    ref = np.zeros((sample.size, cfg.d))
    for n, t in enumerate(sample):
        # token t alone, with the cache cut at its own position
        Ot, _, _ = moa.moa_forward(inp.x[t:t + 1], inp.w_r, None, inp.w_q, inp.k[:, :t + 1], inp.v[:, :t + 1], inp.w_o,
                                   "dense", scale=scale)
        ref[n] = Ot[0]
    err = helpers.rel_err(o[sample], ref)
    say(f"  sampled rel err {err:.3e}")
    assert err <= TOL


# --------------------------------------------------------------------------------------------------
# Dense-training backward (Sec. 3.2, "Dense Training"; gradients of Eq. 7-8, score gradient as in Eq. 3)
# --------------------------------------------------------------------------------------------------
GRADS = (("dx", "dX"), ("dw_r", "dW_r"), ("db_r", "db_r"), ("dw_q", "dW_q"), ("dw_o", "dW_o"), ("dk", "dK"), ("dv", "dV"))


def fwd_bwd(torch, dsmoe, layer, inp, d_out, scale):
    args = [dev(torch, a) for a in (inp.x, inp.w_r, inp.w_q, inp.k, inp.v, inp.w_o)]
    x, w_r, w_q, k, v, w_o = args
    out = layer.fwd(x, w_r, dev(torch, inp.b_r), w_q, k, v, w_o, dsmoe.SEL_ALL, 0, 0.0, float(scale))
    g = layer.bwd(x, w_r, w_q, k, v, w_o, dev(torch, d_out), float(scale))
    torch.cuda.synchronize()
    return out, g


def check_backward(torch, dsmoe, cfg, scale=None, variant=0):
    scale = 1.0 / np.sqrt(cfg.d_head) if scale is None else scale
    inp = gen.make_moa(cfg, variant)
    d_out = gen.make_moa_upstream_grad(cfg, variant)
    say(f"[case] moa backward {cfg.name} T={cfg.T} L={cfg.L} d={cfg.d} E={cfg.E} heads={cfg.n_head}x{cfg.d_head} "
        f"scale={scale:.4f}")
    layer = dsmoe.MoaLayer(cfg.d, cfg.E, cfg.n_head, cfg.d_head, max_tokens=cfg.T)
    out, g = fwd_bwd(torch, dsmoe, layer, inp, d_out, scale)
    O_ref, _, _ = moa.moa_forward(inp.x, inp.w_r, inp.b_r, inp.w_q, inp.k, inp.v, inp.w_o, "dense", scale=scale)
    assert helpers.rel_err(out.float().cpu().numpy(), O_ref) <= TOL
    ref = moa.moa_dense_backward(inp.x, inp.w_r, inp.b_r, inp.w_q, inp.k, inp.v, inp.w_o, d_out, scale)
    for name, rname in GRADS:
        err = helpers.rel_err(g[name].float().cpu().numpy(), ref[rname])
        say(f"  {name}: rel err {err:.3e}")
        assert err <= TOL, name
    return layer, inp, d_out, g


def test_backward_m1_and_bitwise_repeat(torch, dsmoe):
    cfg = gen.MOA_CONFIGS["m1"].with_(mode="dense")
    layer, inp, d_out, g = check_backward(torch, dsmoe, cfg)
    _, g2 = fwd_bwd(torch, dsmoe, layer, inp, d_out, 1.0 / np.sqrt(cfg.d_head))
    for name, _ in GRADS:
        assert torch.equal(g[name], g2[name]), name


@pytest.mark.parametrize("T,L,n_head,d_head", [(1, 1, 2, 64), (1, 37, 1, 128), (129, 129, 2, 64), (300, 555, 2, 128),
                                               (257, 700, 3, 64), (64, 2000, 2, 128), (33, 1000, 4, 64)])
def test_backward_ragged_shapes(torch, dsmoe, T, L, n_head, d_head):
    cfg = gen.MoaConfig("bwd_ragged", 16, T=T, L=L, d=256, E=8, n_head=n_head, d_head=d_head, dtype="bf16", mode="dense",
                        router_std=0.1)
    layer, inp, d_out, g = check_backward(torch, dsmoe, cfg)
    # every product shape of the backward (ragged K steps, K tails from the zero page, causal tile skipping) twice:
    # the hand-counted waits of the contraction core leave no room for run-to-run differences
    _, g2 = fwd_bwd(torch, dsmoe, layer, inp, d_out, 1.0 / np.sqrt(d_head))
    for name, _ in GRADS:
        assert torch.equal(g[name], g2[name]), name


def test_backward_sixteen_and_sixtyfour_experts_and_unit_scale(torch, dsmoe):
    check_backward(torch, dsmoe, gen.MoaConfig("bwd_e16", 17, T=200, L=200, d=512, E=16, n_head=2, d_head=64, dtype="bf16",
                                               mode="dense", router_std=0.1))
    check_backward(torch, dsmoe, gen.MoaConfig("bwd_e64", 18, T=100, L=300, d=256, E=64, n_head=1, d_head=64, dtype="bf16",
                                               mode="dense", router_std=0.1), scale=1.0)


def test_backward_needs_the_matching_dense_forward(torch, dsmoe):
    cfg = gen.MOA_CONFIGS["m1"].with_(mode="dense")
    inp = gen.make_moa(cfg)
    d_out = dev(torch, gen.make_moa_upstream_grad(cfg))
    layer = dsmoe.MoaLayer(cfg.d, cfg.E, cfg.n_head, cfg.d_head, max_tokens=cfg.T)
    x, w_r, w_q, k, v, w_o = [dev(torch, a) for a in (inp.x, inp.w_r, inp.w_q, inp.k, inp.v, inp.w_o)]
    with pytest.raises(dsmoe.DsmoeError) as e:      # no forward yet
        layer.bwd(x, w_r, w_q, k, v, w_o, d_out, 1.0)
    assert e.value.code == dsmoe.ERR_INVALID_ARG
    layer.fwd(x, w_r, None, w_q, k, v, w_o, dsmoe.SEL_TOPK, 2, 0.0, 1.0)
    with pytest.raises(dsmoe.DsmoeError):           # a sparse forward keeps nothing for the backward pass
        layer.bwd(x, w_r, w_q, k, v, w_o, d_out, 1.0)
    layer.fwd(x, w_r, None, w_q, k, v, w_o, dsmoe.SEL_ALL, 0, 0.0, 1.0)
    with pytest.raises(dsmoe.DsmoeError):           # another scale
        layer.bwd(x, w_r, w_q, k, v, w_o, d_out, 0.5)
    layer.bwd(x, w_r, w_q, k, v, w_o, d_out, 1.0)
    torch.cuda.synchronize()


def test_m2_full_size_dense_training_backward(torch, dsmoe):
    """The 6B shape at 2048 tokens, forward and backward; the checker's backward at this size takes a few seconds
    per expert in fp64, so every gradient is compared in full."""
    cfg = gen.MOA_CONFIGS["m2"]
    check_backward(torch, dsmoe, cfg)
