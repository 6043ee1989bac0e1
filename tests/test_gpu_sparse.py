"""GPU parity of the sparse-inference forward (Eq. 1) against the CPU checker, through the C ABI.

Bars: routing objects (selected sets, per-expert counts, dispatch permutation) bit-exact; outputs
within max|gpu - ref| / max|ref| <= 1e-5 (fp32) or 2e-2 (bf16 storage, fp32 accumulation).
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


def weights_to_dev(torch, inp):
    dt = inp.cfg.dtype
    return {k: dev(torch, getattr(inp, k), dt) for k in ("x", "w_r", "b_r", "w_gate", "w_up", "w_down")}


def mode_code(dsmoe, mode):
    return {"topk": dsmoe.SEL_TOPK, "threshold": dsmoe.SEL_THRESHOLD, "threshold_topk": dsmoe.SEL_THRESHOLD_TOPK}[mode]


def mask_to_bool(mask_i64, E):
    m = mask_i64.cpu().numpy().view(np.uint64)
    return ((m[:, None] >> np.arange(E, dtype=np.uint64)[None, :]) & np.uint64(1)).astype(bool)


def run_staged_and_check(torch, dsmoe, inp, mode, k, eps, max_rows=None, materialize=False):
    """Every staged C-ABI call against the matching checker function; returns the GPU output."""
    cfg = inp.cfg
    T, E, tol = inp.x.shape[0], cfg.E, TOL[cfg.dtype]
    say(f"[case] {cfg.name} T={T} d={cfg.d} E={E} f={cfg.f} {cfg.dtype} mode={mode} k={k} eps={eps} "
        f"materialize={materialize}")
    w = weights_to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, E, cfg.dtype, max_tokens=max(T, 1), max_rows=max_rows,
                        expert="gelu" if inp.w_up is None else "swiglu")

    S_ref = orc.route(inp.x, inp.w_r, inp.b_r)
    M_ref = orc.select(S_ref, mode, k, eps)
    r_ref = orc.dispatch(M_ref, S_ref)

    # route
    probs = layer.route(w["x"], w["w_r"], w["b_r"])
    torch.cuda.synchronize()
    S_gpu = probs.cpu().numpy()
    assert helpers.rel_err(S_gpu, S_ref) <= 1e-5
    np.testing.assert_allclose(S_gpu.sum(axis=1), 1.0, atol=1e-5)

    # select: on the GPU's own fp32 probabilities, checker decides on the same fp32 values
    mask, cnt = layer.select(probs, mode_code(dsmoe, mode), k, eps)
    M_same = orc.select(S_gpu, mode, k, np.float32(eps))
    M_gpu = mask_to_bool(mask, E)
    np.testing.assert_array_equal(M_gpu, M_same)
    np.testing.assert_array_equal(cnt.cpu().numpy(), M_same.sum(axis=1))
    # margin-conditioned inputs: the sets also equal the fp64 decision
    np.testing.assert_array_equal(M_gpu, M_ref)

    # dispatch
    r = layer.dispatch(w["x"], probs, mask, materialize=materialize)
    assert layer.poll_error() == dsmoe.OK
    r_same = orc.dispatch(M_gpu, S_gpu)
    nnz = int(r["nnz"][0].item())
    assert nnz == r_same.nnz == r_ref.nnz
    np.testing.assert_array_equal(r["expert_off"].cpu().numpy(), r_same.expert_off)
    np.testing.assert_array_equal(r["row_token"].cpu().numpy()[:nnz], r_same.row_token)
    np.testing.assert_array_equal(r["tok_off"].cpu().numpy(), r_same.tok_off)
    np.testing.assert_array_equal(r["tok_rows"].cpu().numpy()[:nnz], r_same.tok_rows)
    np.testing.assert_array_equal(r["row_weight"].cpu().numpy()[:nnz], r_same.row_weight)
    np.testing.assert_array_equal(r["row_token"].cpu().numpy()[:nnz], r_ref.row_token)
    if materialize:
        xp = r["x_perm"][:nnz].float().cpu().numpy()
        np.testing.assert_array_equal(xp, inp.x[r_same.row_token])

    # expert FFN on the dispatched rows
    y = layer.expert_ffn(w["x"], r, w["w_gate"], w["w_up"], w["w_down"])
    torch.cuda.synchronize()
    Y_ref = orc.expert_outputs_permuted(inp.x, r_ref, inp.w_gate, inp.w_up, inp.w_down)
    y_gpu = y[:nnz].float().cpu().numpy()
    if nnz:
        assert helpers.rel_err(y_gpu, Y_ref) <= tol

    # combine
    out = layer.combine(y, r, T)
    torch.cuda.synchronize()
    O_ref, _, _ = orc.sparse_forward(inp.x, inp.w_r, inp.b_r, inp.w_gate, inp.w_up, inp.w_down, mode, k, eps)
    o_gpu = out.float().cpu().numpy()
    if T:
        assert helpers.rel_err(o_gpu, O_ref) <= tol
        # the combine alone, on the GPU's own rows, in fp64
        O_cmb = orc.combine(y_gpu.astype(np.float64), r_same, T)
        assert helpers.rel_err(o_gpu, O_cmb) <= (1e-6 if cfg.dtype == "f32" else 6e-3)

    # fused call gives the same routing and (bitwise) the same output
    out2 = layer.sparse_fwd(w["x"], w["w_r"], w["b_r"], w["w_gate"], w["w_up"], w["w_down"],
                            mode_code(dsmoe, mode), k, eps)
    assert layer.poll_error() == dsmoe.OK
    p2, m2, eo2, rt2 = layer.sparse_fwd_routing(T)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(mask_to_bool(m2, E), M_ref)
    np.testing.assert_array_equal(eo2.cpu().numpy(), r_ref.expert_off)
    np.testing.assert_array_equal(rt2.cpu().numpy()[:nnz], r_ref.row_token)
    if cfg.dtype == "bf16" and 0 < T <= 128:
        # decode-sized batches take the weight-streaming kernels (fp32 partial sums, one final rounding)
        err2 = helpers.rel_err(out2.float().cpu().numpy(), O_ref)
        say(f"  weight-streaming path rel err {err2:.3e}")
        assert err2 <= tol
    else:
        assert torch.equal(out2, out)
    return o_gpu


def conditioned(cfg, mode, k, eps, variant=0):
    inp = gen.make_layer(cfg, variant)
    helpers.condition_margins(inp, mode, k, eps)
    return inp


# --------------------------------------------------------------------------------------------------
def test_c1_tiny_fp32_topk2(torch, dsmoe):
    cfg = gen.CONFIGS["c1"]
    run_staged_and_check(torch, dsmoe, conditioned(cfg, "topk", 2, 0.0), "topk", 2, 0.0)


def test_c1_threshold_and_materialised_permutation(torch, dsmoe):
    cfg = gen.CONFIGS["c1"].with_(router_std=0.1)
    run_staged_and_check(torch, dsmoe, conditioned(cfg, "threshold", 0, 0.1), "threshold", 0, 0.1, materialize=True)


def test_c1_dense_limits_k_equals_E_and_eps_zero(torch, dsmoe):
    cfg = gen.CONFIGS["c1"]
    inp = gen.make_layer(cfg, 0)
    o1 = run_staged_and_check(torch, dsmoe, inp, "topk", cfg.E, 0.0)
    o2 = run_staged_and_check(torch, dsmoe, inp, "threshold", 0, 0.0)
    D, _, _ = orc.dense_forward(inp.x, inp.w_r, inp.b_r, inp.w_gate, inp.w_up, inp.w_down)
    assert helpers.rel_err(o1, D) <= 1e-5 and helpers.rel_err(o2, D) <= 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode,k,eps", [("topk", 3, 0.0), ("threshold", 0, 0.05)])
def test_ragged_multi_tile(torch, dsmoe, dtype, mode, k, eps):
    # T not a multiple of any tile, d_ff with a ragged column tile, several row tiles per expert
    cfg = gen.LayerConfig("ragged", 11, T=777, d=320, E=16, f=192, dtype=dtype, mode=mode, k=k, eps=eps,
                          router_std=0.08)
    run_staged_and_check(torch, dsmoe, conditioned(cfg, mode, k, eps), mode, k, eps)


@pytest.mark.parametrize("name,T,dtype,eps", [("c1", 128, "f32", 0.11), ("c2", 300, "bf16", 0.02),
                                              ("c2", 32, "bf16", 0.02), ("c2", 128, "bf16", 0.05)])
def test_threshold_topk_selection(torch, dsmoe, name, T, dtype, eps):
    """Sec. 4.3: K = batch mean of the threshold counts (rounded half up), then top-K; staged and fused,
    prefill-sized and decode-sized."""
    base = gen.CONFIGS[name]
    d = base.d if name == "c1" else 512
    cfg = base.with_(name=f"ttk_{name}_{T}", index=12, T=T, d=d, f=base.f if name == "c1" else 128, dtype=dtype,
                     mode="threshold", eps=eps, router_std=base.router_std if name == "c1" else 1.5 / np.sqrt(d))
    inp = conditioned(cfg, "threshold_topk", 0, eps)
    K = orc.threshold_topk_k(orc.route(inp.x, inp.w_r, inp.b_r), eps)
    say(f"  Threshold-TopK: K = {K}")
    assert 1 <= K < cfg.E
    run_staged_and_check(torch, dsmoe, inp, "threshold_topk", 0, eps)


@pytest.mark.parametrize("T,E", [(300, 24), (64, 24), (500, 32)])
def test_normalised_threshold_of_the_paper(torch, dsmoe, T, E):
    """Sec. 4.2 (footnote): the paper thresholds the normalised probability N * S_i.  With DSMOE_SEL_NORMALISED
    the caller passes that value; the selection must equal the checker's raw-probability rule at eps / N (the
    quotient in fp32, as the library forms it), staged and fused, prefill- and decode-sized."""
    eps_paper = 0.48                                   # the paper's example value (Sec. 4.3)
    raw = np.float32(eps_paper) / np.float32(E)
    d = 256
    cfg = gen.LayerConfig("norm_eps", 17, T=T, d=d, E=E, f=128, dtype="bf16", mode="threshold", eps=float(raw),
                          router_std=1.5 / np.sqrt(d))
    inp = conditioned(cfg, "threshold", 0, float(raw))
    say(f"[case] normalised threshold {eps_paper} on {E} experts = raw {raw:.6f}, T={T}")
    w = weights_to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, E, "bf16", max_tokens=T)
    norm = dsmoe.SEL_THRESHOLD | dsmoe.SEL_NORMALISED
    probs = layer.route(w["x"], w["w_r"], None)
    mask, cnt = layer.select(probs, norm, 0, eps_paper)
    S_gpu = probs.cpu().numpy()
    M_same = orc.select_threshold(S_gpu, raw)
    np.testing.assert_array_equal(mask_to_bool(mask, E), M_same)
    np.testing.assert_array_equal(cnt.cpu().numpy(), M_same.sum(axis=1))
    M_ref = orc.select_threshold(orc.route(inp.x, inp.w_r, None), float(raw))
    np.testing.assert_array_equal(M_same, M_ref)
    assert 1.0 < M_ref.sum(axis=1).mean() < E - 1       # the rule is neither trivial nor dense here
    out_n = layer.sparse_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], norm, 0, eps_paper).clone()
    _, m_n, _, _ = layer.sparse_fwd_routing(T)
    np.testing.assert_array_equal(mask_to_bool(m_n, E), M_ref)
    out_r = layer.sparse_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], dsmoe.SEL_THRESHOLD, 0,
                             float(raw))
    assert layer.poll_error() == dsmoe.OK
    assert torch.equal(out_n, out_r)
    O_ref, _, _ = orc.sparse_forward(inp.x, inp.w_r, None, inp.w_gate, inp.w_up, inp.w_down, "threshold", 0, float(raw))
    assert helpers.rel_err(out_n.float().cpu().numpy(), O_ref) <= TOL["bf16"]
    # Threshold-TopK with the normalised threshold: K from the same counts
    mask_t, _ = layer.select(probs, dsmoe.SEL_THRESHOLD_TOPK | dsmoe.SEL_NORMALISED, 0, eps_paper)
    K = orc.threshold_topk_k(S_gpu, raw)
    np.testing.assert_array_equal(mask_to_bool(mask_t, E), orc.select_topk(S_gpu, K))


@pytest.mark.parametrize("name,T,dtype,mode,k,eps,materialize", [
    ("c1", 128, "f32", "topk", 2, 0.0, False), ("c1", 128, "f32", "threshold", 0, 0.13, True),
    ("rag", 777, "bf16", "threshold", 0, 0.05, False), ("rag", 777, "f32", "topk", 3, 0.0, False),
    ("rag", 40, "bf16", "topk", 3, 0.0, True), ("rag", 128, "bf16", "threshold", 0, 0.05, False),
    ("rag", 1, "bf16", "topk", 4, 0.0, False)])
def test_gelu_two_matrix_expert(torch, dsmoe, name, T, dtype, mode, k, eps, materialize):
    """The paper's own expert (Sec. 4.1): e(x) = gelu(x W_1) W_2, through every staged call and the fused one."""
    if name == "c1":
        cfg = gen.CONFIGS["c1"].with_(name="c1_gelu", mode=mode, k=k, eps=eps)
    else:
        cfg = gen.LayerConfig("ragged_gelu", 13, T=T, d=320, E=16, f=192, dtype=dtype, mode=mode, k=k, eps=eps,
                              router_std=0.08)
    inp = conditioned(cfg, mode, k, eps)
    inp.w_up = None
    run_staged_and_check(torch, dsmoe, inp, mode, k, eps, materialize=materialize)


@pytest.mark.parametrize("expert", ["swiglu", "gelu"])
@pytest.mark.parametrize("counts", [
    [0, 1, 127, 128, 129, 255, 256, 257, 0, 384, 385, 640, 2, 200, 513, 0],   # every remainder class of both heights
    [300] * 40 + [5] * 3 + [0] * 5,                                   # full and half tiles on most experts
    [130] * 8,                                                        # few full tiles: cut in halves
])
def test_expert_ffn_on_crafted_row_groups(torch, dsmoe, counts, expert):
    """The grouped FFN alone on hand-made row groups (sizes around the kernels' 128- and 256-row tiles), each
    expert's rows against the checker's plain FFN of that expert (Eq. 1, the e_i(X) factor)."""
    E, d, f, T = len(counts), 256, 192, 700
    cfg = gen.LayerConfig("groups", 31, T=T, d=d, E=E, f=f, dtype="bf16", mode="topk", k=1, router_std=0.05)
    inp = gen.make_layer(cfg, 0)
    if expert == "gelu":
        inp.w_up = None
    rng = np.random.default_rng(5)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    nnz = int(off[-1])
    row_token = rng.integers(0, T, size=nnz).astype(np.int32)
    say(f"[case] crafted groups E={E} nnz={nnz} expert={expert}")
    w = weights_to_dev(torch, inp)
    # a row capacity well above nnz gives a grid with idle blocks, which is when full tiles are cut in halves
    layer = dsmoe.Layer(d, f, E, "bf16", max_tokens=4096, max_rows=max(nnz, 20000), expert=expert)
    for materialize in (False, True):
        r = dict(expert_off=torch.from_numpy(off).cuda(), row_token=torch.from_numpy(row_token).cuda())
        if materialize:
            r["x_perm"] = w["x"][torch.from_numpy(row_token.astype(np.int64)).cuda()].contiguous()
        y = layer.expert_ffn(w["x"], r, w["w_gate"], w["w_up"], w["w_down"])
        torch.cuda.synchronize()
        y_gpu = y[:nnz].float().cpu().numpy()
        for e in range(E):
            if counts[e] == 0:
                continue
            rows = row_token[off[e]:off[e + 1]]
            ref = orc.expert_ffn(inp.x[rows], inp.w_gate[e], None if inp.w_up is None else inp.w_up[e], inp.w_down[e])
            assert helpers.rel_err(y_gpu[off[e]:off[e + 1]], ref) <= TOL["bf16"], (e, counts[e], materialize)


@pytest.mark.parametrize("counts", [[130] * 8, [300, 20, 0, 257, 5, 128, 129, 1]])
def test_expert_ffn_long_contraction_few_tiles(torch, dsmoe, counts):
    """Few row tiles and a long contraction (d = 2048, 64 K steps: the chained pipeline and the half tiles of an
    uneven last turn); twice, bitwise equal."""
    E, d, f, T = len(counts), 2048, 192, 400
    cfg = gen.LayerConfig("ksplit", 32, T=T, d=d, E=E, f=f, dtype="bf16", mode="topk", k=1, router_std=0.05)
    inp = gen.make_layer(cfg, 0)
    rng = np.random.default_rng(6)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    nnz = int(off[-1])
    row_token = rng.integers(0, T, size=nnz).astype(np.int32)
    say(f"[case] long contraction, few tiles: E={E} nnz={nnz}")
    w = weights_to_dev(torch, inp)
    layer = dsmoe.Layer(d, f, E, "bf16", max_tokens=4096, max_rows=20000)
    r = dict(expert_off=torch.from_numpy(off).cuda(), row_token=torch.from_numpy(row_token).cuda())
    y1 = layer.expert_ffn(w["x"], r, w["w_gate"], w["w_up"], w["w_down"]).clone()
    y2 = layer.expert_ffn(w["x"], r, w["w_gate"], w["w_up"], w["w_down"])
    torch.cuda.synchronize()
    assert torch.equal(y1[:nnz], y2[:nnz])
    y_gpu = y2[:nnz].float().cpu().numpy()
    for e in range(E):
        if counts[e] == 0:
            continue
        rows = row_token[off[e]:off[e + 1]]
        ref = orc.expert_ffn(inp.x[rows], inp.w_gate[e], inp.w_up[e], inp.w_down[e])
        assert helpers.rel_err(y_gpu[off[e]:off[e + 1]], ref) <= TOL["bf16"], (e, counts[e])


def test_skewed_router_bias_empty_and_hot_experts(torch, dsmoe):
    cfg = gen.LayerConfig("skew", 12, T=500, d=256, E=24, f=128, dtype="bf16", mode="threshold", eps=0.04,
                          router_std=0.05, zipf_s=2.0)
    inp = conditioned(cfg, "threshold", 0, 0.04)
    S = orc.route(inp.x, inp.w_r, inp.b_r)
    cnt = orc.select_threshold(S, 0.04).sum(axis=0)
    assert cnt.max() > 400 and cnt.min() == 0          # one expert takes nearly every token, some none
    run_staged_and_check(torch, dsmoe, inp, "threshold", 0, 0.04)


def test_one_hot_router_sends_everything_to_one_expert(torch, dsmoe):
    cfg = gen.LayerConfig("onehot", 13, T=200, d=128, E=8, f=64, dtype="f32", mode="topk", k=1, router_std=0.0)
    inp = gen.make_layer(cfg, 0)
    inp.b_r = np.zeros(8, dtype=np.float32)
    inp.b_r[5] = 60.0
    o = run_staged_and_check(torch, dsmoe, inp, "topk", 1, 0.0)
    ref = orc.expert_ffn(inp.x, inp.w_gate[5], inp.w_up[5], inp.w_down[5])
    assert helpers.rel_err(o, ref) <= 1e-5


def test_exact_ties_from_duplicated_router_columns(torch, dsmoe):
    cfg = gen.LayerConfig("ties", 14, T=256, d=128, E=8, f=64, dtype="bf16", mode="topk", k=2, router_std=0.1)
    inp = gen.make_layer(cfg, 0)
    inp.w_r[:, 6] = inp.w_r[:, 1]
    inp.w_r[:, 3] = inp.w_r[:, 1]
    w = weights_to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=cfg.T)
    probs = layer.route(w["x"], w["w_r"], None)
    S = probs.cpu().numpy()
    assert np.array_equal(S[:, 1], S[:, 3]) and np.array_equal(S[:, 1], S[:, 6])
    for k in (1, 2, 3):
        mask, _ = layer.select(probs, dsmoe.SEL_TOPK, k, 0.0)
        np.testing.assert_array_equal(mask_to_bool(mask, cfg.E), orc.select_topk(S, k))
    # threshold fallback with ties: eps above every probability -> arg-max, lowest index
    mask, cnt = layer.select(probs, dsmoe.SEL_THRESHOLD, 0, 0.999)
    np.testing.assert_array_equal(mask_to_bool(mask, cfg.E), orc.select_threshold(S, np.float32(0.999)))
    assert (cnt.cpu().numpy() == 1).all()


@pytest.mark.parametrize("T", [0, 1, 8, 32, 128])
@pytest.mark.parametrize("mode,k,eps", [("topk", 4, 0.0), ("threshold", 0, 0.02)])
def test_c3_decode_sizes(torch, dsmoe, T, mode, k, eps):
    cfg = gen.CONFIGS["c3"].with_(T=T, E=32)
    inp = gen.make_layer(cfg, T)
    if T:
        helpers.condition_margins(inp, mode, k, eps)
    run_staged_and_check(torch, dsmoe, inp, mode, k, eps, max_rows=T * 32)


@pytest.mark.parametrize("T,d,E,f,mode,k,eps,zipf", [
    (128, 320, 16, 192, "threshold", 0, 0.0, 0.0),     # every expert on every token; ragged column slices
    (128, 256, 64, 64, "topk", 2, 0.0, 3.0),           # 64 experts, a few of them take nearly all tokens
    (100, 512, 8, 256, "topk", 1, 0.0, 0.0),
    (3, 2048, 32, 512, "topk", 1, 0.0, 0.0),           # at most three active experts: deepest K split
    (65, 192, 8, 64, "threshold", 0, 0.1, 0.0),
])
def test_weight_streaming_path_shapes(torch, dsmoe, T, d, E, f, mode, k, eps, zipf):
    cfg = gen.LayerConfig("decode", 16, T=T, d=d, E=E, f=f, dtype="bf16", mode=mode, k=k, eps=eps,
                          router_std=1.0 / np.sqrt(d), zipf_s=zipf)
    run_staged_and_check(torch, dsmoe, conditioned(cfg, mode, k, eps), mode, k, eps)


def test_weight_streaming_path_overflow_and_repeatability(torch, dsmoe):
    cfg = gen.CONFIGS["c3"].with_(T=64)
    inp = conditioned(cfg, "topk", 4, 0.0)
    w = weights_to_dev(torch, inp)
    args = (w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], dsmoe.SEL_TOPK, 4, 0.0)
    small = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=64, max_rows=200)    # needs 256 rows
    out = small.sparse_fwd(*args)
    assert small.poll_error() == dsmoe.ERR_CAPACITY
    _, _, eo, _ = small.sparse_fwd_routing(64)
    assert int(eo.abs().sum().item()) == 0 and float(out.float().abs().max().item()) == 0.0
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=64)
    outs = [layer.sparse_fwd(*args).clone() for _ in range(3)]
    assert layer.poll_error() == dsmoe.OK
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    O, _, _ = orc.sparse_forward(inp.x, inp.w_r, None, inp.w_gate, inp.w_up, inp.w_down, "topk", 4)
    assert helpers.rel_err(outs[0].float().cpu().numpy(), O) <= TOL["bf16"]


def test_all_expert_decode_kernel_alternating_inputs_and_bounded_waits(torch, dsmoe):
    """The persistent decode kernel (8 .. 64 tokens that select nearly every expert) hands results between
    blocks through counters that each call must leave reset: alternate two different inputs and two batch sizes
    many times on one context and require bitwise the results of the first round; then make every wait between
    blocks give up at once (spin limit 0): the kernel must still end, the deferred status must say so, and the
    next call must be right again."""
    cfg = gen.CONFIGS["c3"].with_(T=64)
    a = conditioned(cfg, "topk", 4, 0.0, variant=1)
    b = conditioned(cfg.with_(T=40), "threshold", 0, 0.02, variant=2)
    wa, wb = weights_to_dev(torch, a), weights_to_dev(torch, b)
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=128)
    assert dsmoe.dense_decode_applies(layer, 64, dsmoe.SEL_TOPK, 4, 0.0)
    assert dsmoe.dense_decode_applies(layer, 40, dsmoe.SEL_THRESHOLD, 0, 0.02)
    call_a = lambda: layer.sparse_fwd(wa["x"], wa["w_r"], None, wa["w_gate"], wa["w_up"], wa["w_down"], dsmoe.SEL_TOPK, 4, 0.0)
    call_b = lambda: layer.sparse_fwd(wb["x"], wb["w_r"], None, wb["w_gate"], wb["w_up"], wb["w_down"],
                                      dsmoe.SEL_THRESHOLD, 0, 0.02)
    ref_a, ref_b = call_a().clone(), call_b().clone()
    assert layer.poll_error() == dsmoe.OK
    Oa, _, _ = orc.sparse_forward(a.x, a.w_r, None, a.w_gate, a.w_up, a.w_down, "topk", 4)
    Ob, _, _ = orc.sparse_forward(b.x, b.w_r, None, b.w_gate, b.w_up, b.w_down, "threshold", 0, 0.02)
    assert helpers.rel_err(ref_a.float().cpu().numpy(), Oa) <= TOL["bf16"]
    assert helpers.rel_err(ref_b.float().cpu().numpy(), Ob) <= TOL["bf16"]
    for i in range(40):                                   # back to back, no synchronisation in between
        oa, ob = call_a(), call_b()
        if i % 8 == 7:
            assert torch.equal(oa, ref_a) and torch.equal(ob, ref_b), i
    assert torch.equal(oa, ref_a) and torch.equal(ob, ref_b)
    assert layer.poll_error() == dsmoe.OK
    # every wait gives up at once: the call ends, is reported, and leaves the context usable
    layer.set_sync_spin_limit(0)
    call_a()
    torch.cuda.synchronize()
    assert layer.poll_error() == dsmoe.ERR_INTERNAL
    assert b"gave up" in layer.lib.dsmoe_last_error(layer.ctx)
    layer.set_sync_spin_limit(1 << 20)
    assert torch.equal(call_a(), ref_a)
    assert layer.poll_error() == dsmoe.OK


def test_capacity_overflow_is_reported_and_harmless(torch, dsmoe):
    cfg = gen.CONFIGS["c1"]
    inp = gen.make_layer(cfg, 0)
    w = weights_to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=cfg.T, max_rows=200)   # needs 256 rows
    out = layer.sparse_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], dsmoe.SEL_TOPK, 2, 0.0)
    assert layer.poll_error() == dsmoe.ERR_CAPACITY
    assert layer.poll_error() == dsmoe.OK                      # the flag is cleared by the poll
    _, _, eo, _ = layer.sparse_fwd_routing(cfg.T)
    assert int(eo.abs().sum().item()) == 0                     # empty routing was published
    assert float(out.abs().max().item()) == 0.0                # combine of nothing
    # a call that fits still works afterwards
    out = layer.sparse_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], dsmoe.SEL_TOPK, 1, 0.0)
    assert layer.poll_error() == dsmoe.OK
    O, _, _ = orc.sparse_forward(inp.x, inp.w_r, None, inp.w_gate, inp.w_up, inp.w_down, "topk", 1)
    assert helpers.rel_err(out.float().cpu().numpy(), O) <= 1e-5


def test_dispatch_ignores_mask_bits_above_the_expert_count(torch, dsmoe):
    """A caller's selection mask may carry stray bits at or above E: the dispatch drops them, so counts, offsets
    and rows equal those of the clean masks (and no row index passes nnz)."""
    cfg = gen.LayerConfig("stray", 18, T=700, d=64, E=24, f=64, dtype="bf16", mode="topk", k=3, router_std=0.1)
    inp = gen.make_layer(cfg, 0)
    S = orc.route(inp.x, inp.w_r, None).astype(np.float32)
    M = orc.select_topk(S, 3)
    r_ref = orc.dispatch(M, S)
    bits = (M.astype(np.uint64) << np.arange(cfg.E, dtype=np.uint64)[None, :]).sum(axis=1, dtype=np.uint64)
    rng = np.random.default_rng(3)
    stray = rng.integers(0, 1 << 40, size=cfg.T, dtype=np.uint64) << np.uint64(cfg.E)
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, "bf16", max_tokens=cfg.T, max_rows=r_ref.nnz)   # no spare row
    x = torch.from_numpy(inp.x).cuda().to(torch.bfloat16)
    probs = torch.from_numpy(S).cuda()
    clean = layer.dispatch(x, probs, torch.from_numpy(bits.view(np.int64)).cuda())
    dirty = layer.dispatch(x, probs, torch.from_numpy((bits | stray).view(np.int64)).cuda())
    assert layer.poll_error() == dsmoe.OK
    for k in ("expert_off", "row_token", "row_weight", "tok_off", "tok_rows", "nnz"):
        n = r_ref.nnz if k in ("row_token", "row_weight", "tok_rows") else (1 if k == "nnz" else clean[k].numel())
        assert torch.equal(clean[k][:n], dirty[k][:n]), k
    np.testing.assert_array_equal(dirty["expert_off"].cpu().numpy(), r_ref.expert_off)
    np.testing.assert_array_equal(dirty["tok_rows"].cpu().numpy()[:r_ref.nnz], r_ref.tok_rows)


def test_repeated_calls_are_bitwise_identical(torch, dsmoe):
    cfg = gen.LayerConfig("det", 15, T=1000, d=256, E=16, f=128, dtype="bf16", mode="threshold", eps=0.05,
                          router_std=0.08)
    inp = gen.make_layer(cfg, 0)
    w = weights_to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, cfg.dtype, max_tokens=cfg.T)
    outs = [layer.sparse_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"],
                             dsmoe.SEL_THRESHOLD, 0, 0.05).clone() for _ in range(3)]
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


# --------------------------------------------------------------------------------------------------
# full benchmark sizes, in the launch configuration bench.py times (dsmoe_sparse_fwd)
# --------------------------------------------------------------------------------------------------
def full_size_check(torch, dsmoe, name, n_sample, max_rows, cfg=None):
    """n_sample = None: every output row is compared (the checker runs the whole layer)."""
    cfg = gen.CONFIGS[name] if cfg is None else cfg
    say(f"[case] full-size {name}: generating inputs")
    inp = conditioned(cfg, cfg.mode, cfg.k, cfg.eps)
    T, E = cfg.T, cfg.E
    S_ref = orc.route(inp.x, inp.w_r, inp.b_r)
    M_ref = orc.select(S_ref, cfg.mode, cfg.k, cfg.eps)
    r_ref = orc.dispatch(M_ref, S_ref)
    say(f"[case] full-size {name}: nnz={r_ref.nnz} mean active={r_ref.nnz / T:.2f} "
        f"rows/expert min={r_ref.cnt_exp.min()} max={r_ref.cnt_exp.max()}")
    assert r_ref.nnz <= max_rows
    w = weights_to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, E, cfg.dtype, max_tokens=T, max_rows=max_rows)
    out = layer.sparse_fwd(w["x"], w["w_r"], w["b_r"], w["w_gate"], w["w_up"], w["w_down"],
                           mode_code(dsmoe, cfg.mode), cfg.k, cfg.eps)
    assert layer.poll_error() == dsmoe.OK
    probs, mask, eo, rt = layer.sparse_fwd_routing(T)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(mask_to_bool(mask, E), M_ref)
    np.testing.assert_array_equal(eo.cpu().numpy(), r_ref.expert_off)
    np.testing.assert_array_equal(rt.cpu().numpy()[:r_ref.nnz], r_ref.row_token)
    assert helpers.rel_err(probs.cpu().numpy(), S_ref) <= 1e-5
    if n_sample is None:
        tokens = np.arange(T)
    else:     # sampled output rows (each token's output depends on no other token)
        g = np.random.default_rng(cfg.index)
        tokens = np.sort(g.choice(T, size=n_sample, replace=False))
        tokens[0], tokens[-1] = 0, T - 1
    O_ref, _, _ = orc.sparse_forward(inp.x, inp.w_r, inp.b_r, inp.w_gate, inp.w_up, inp.w_down, cfg.mode,
                                     cfg.k, cfg.eps, tokens=tokens)
    o = out.float().cpu().numpy()
    err = helpers.rel_err(o[tokens], O_ref)
    say(f"[case] full-size {name}: rel err over {tokens.size} of {T} output rows {err:.3e}")
    assert err <= TOL[cfg.dtype]
    assert np.isfinite(o).all()
    return r_ref


def test_c2_full_size_sparse_prefill(torch, dsmoe):
    r = full_size_check(torch, dsmoe, "c2", n_sample=None, max_rows=4096 * 16)
    assert 0.30 < r.nnz / (4096 * 32) < 0.42


def test_c5_full_size_skewed_prefill(torch, dsmoe):
    r = full_size_check(torch, dsmoe, "c5", n_sample=None, max_rows=16384 * 24)
    assert r.cnt_exp.max() > 10 * r.cnt_exp.min()


@pytest.mark.parametrize("T", [512, 96])
def test_largest_layer_of_the_paper(torch, dsmoe, T):
    """The expert layer of the largest model in the paper's speed test (Table 6: embedding 7168, 32 experts of
    hidden width 896, top-4), as a prefill-sized call (grouped kernels) and a decode-sized one (weight-streaming
    kernels); sampled output rows against the checker."""
    cfg = gen.LayerConfig(f"ds_moe_19b_T{T}", 15, T=T, d=7168, E=32, f=896, dtype="bf16", mode="topk", k=4,
                          router_std=1.5 / np.sqrt(7168))
    full_size_check(torch, dsmoe, cfg.name, n_sample=min(T, 64), max_rows=4 * T, cfg=cfg)


# --------------------------------------------------------------------------------------------------
# at most 4 tokens: the three few-token kernels (router included, weight rows through the vector ALUs)
# --------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("T,d,E,f,mode,k,eps,expert", [
    (1, 2048, 32, 512, "topk", 4, 0.0, "swiglu"),
    (1, 2048, 32, 512, "topk", 1, 0.0, "swiglu"),          # one active expert: its rows spread over every block
    (2, 7168, 32, 896, "threshold", 0, 0.03, "swiglu"),    # the largest layer of the paper: two chunks of a W_down row per thread
    (3, 2048, 32, 512, "threshold", 0, 0.02, "swiglu"),
    (4, 256, 64, 64, "topk", 2, 0.0, "swiglu"),            # 64 experts, narrow rows: many rows per pass
    (3, 512, 8, 4096, "topk", 1, 0.0, "swiglu"),           # one weight row per pass
    (4, 4096, 16, 128, "topk", 3, 0.0, "swiglu"),
    (4, 1024, 16, 256, "topk", 2, 0.0, "gelu"),
    (2, 1024, 16, 256, "threshold", 0, 0.05, "gelu"),
])
def test_few_token_kernels(torch, dsmoe, T, d, E, f, mode, k, eps, expert):
    cfg = gen.LayerConfig("few", 19, T=T, d=d, E=E, f=f, dtype="bf16", mode=mode, k=k, eps=eps,
                          router_std=1.5 / np.sqrt(d))
    inp = conditioned(cfg, mode, k, eps, variant=T)
    if expert == "gelu":
        inp.w_up = None
    say(f"[case] few tokens T={T} d={d} E={E} f={f} {mode} k={k} eps={eps} {expert}")
    w = weights_to_dev(torch, inp)
    layer = dsmoe.Layer(d, f, E, "bf16", max_tokens=T, expert=expert)
    code = mode_code(dsmoe, mode)
    assert dsmoe.sparse_fwd_path(layer, T, code, k, eps) == dsmoe.PATH_FEW_TOKENS
    args = (w["x"], w["w_r"], w["b_r"], w["w_gate"], w["w_up"], w["w_down"], code, k, eps)
    out = layer.sparse_fwd(*args).clone()
    assert layer.poll_error() == dsmoe.OK
    probs, mask, eo, rt = layer.sparse_fwd_routing(T)
    torch.cuda.synchronize()
    O_ref, S_ref, M_ref = orc.sparse_forward(inp.x, inp.w_r, inp.b_r, inp.w_gate, inp.w_up, inp.w_down, mode, k, eps)
    assert helpers.rel_err(probs.cpu().numpy(), S_ref) <= 1e-5
    np.testing.assert_array_equal(mask_to_bool(mask, E), M_ref)
    r_ref = orc.dispatch(M_ref, S_ref)
    np.testing.assert_array_equal(eo.cpu().numpy(), r_ref.expert_off)
    np.testing.assert_array_equal(rt.cpu().numpy()[:r_ref.nnz], r_ref.row_token)
    err = helpers.rel_err(out.float().cpu().numpy(), O_ref)
    say(f"  rel err {err:.3e}")
    assert err <= TOL["bf16"]
    for _ in range(2):                                         # bitwise reproducible
        assert torch.equal(layer.sparse_fwd(*args), out)


def test_few_token_kernels_threshold_nobody_reaches_and_overflow(torch, dsmoe):
    cfg = gen.CONFIGS["c3"].with_(T=4, E=32)
    inp = gen.make_layer(cfg, 3)
    w = weights_to_dev(torch, inp)
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, "bf16", max_tokens=4)
    # a threshold no score reaches: every token keeps its best expert alone
    out = layer.sparse_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], dsmoe.SEL_THRESHOLD, 0, 0.99)
    assert layer.poll_error() == dsmoe.OK
    _, mask, _, _ = layer.sparse_fwd_routing(4)
    O, S, M = orc.sparse_forward(inp.x, inp.w_r, None, inp.w_gate, inp.w_up, inp.w_down, "threshold", 0, 0.99)
    assert (M.sum(axis=1) == 1).all()
    np.testing.assert_array_equal(mask_to_bool(mask, cfg.E), M)
    assert helpers.rel_err(out.float().cpu().numpy(), O) <= TOL["bf16"]
    # more selected pairs than rows: reported, output zero, and the next call is fine
    small = dsmoe.Layer(cfg.d, cfg.f, cfg.E, "bf16", max_tokens=4, max_rows=10)
    out = small.sparse_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], dsmoe.SEL_TOPK, 4, 0.0)
    assert small.poll_error() == dsmoe.ERR_CAPACITY
    assert float(out.float().abs().max().item()) == 0.0
    out = small.sparse_fwd(w["x"], w["w_r"], None, w["w_gate"], w["w_up"], w["w_down"], dsmoe.SEL_TOPK, 2, 0.0)
    assert small.poll_error() == dsmoe.OK
    O, _, _ = orc.sparse_forward(inp.x, inp.w_r, None, inp.w_gate, inp.w_up, inp.w_down, "topk", 2)
    assert helpers.rel_err(out.float().cpu().numpy(), O) <= TOL["bf16"]


def test_few_token_kernels_with_router_bias_and_smallest_layer(torch, dsmoe):
    """A skewed router (bias per expert) through the in-kernel router, and the smallest layer the library accepts."""
    for T, d, E, f, zipf in ((3, 1024, 32, 256, 1.5), (2, 64, 8, 64, 0.0), (4, 64, 64, 64, 2.0)):
        cfg = gen.LayerConfig("few_bias", 24, T=T, d=d, E=E, f=f, dtype="bf16", mode="topk", k=2, eps=0.0,
                              router_std=1.0 / np.sqrt(d), zipf_s=zipf)
        inp = conditioned(cfg, "topk", 2, 0.0, variant=T)
        assert (inp.b_r is not None) == (zipf > 0)
        w = weights_to_dev(torch, inp)
        layer = dsmoe.Layer(d, f, E, "bf16", max_tokens=T)
        assert dsmoe.sparse_fwd_path(layer, T, dsmoe.SEL_TOPK, 2, 0.0) == dsmoe.PATH_FEW_TOKENS
        out = layer.sparse_fwd(w["x"], w["w_r"], w["b_r"], w["w_gate"], w["w_up"], w["w_down"], dsmoe.SEL_TOPK, 2, 0.0)
        assert layer.poll_error() == dsmoe.OK
        _, mask, _, _ = layer.sparse_fwd_routing(T)
        O, S, M = orc.sparse_forward(inp.x, inp.w_r, inp.b_r, inp.w_gate, inp.w_up, inp.w_down, "topk", 2, 0.0)
        np.testing.assert_array_equal(mask_to_bool(mask, E), M)
        assert helpers.rel_err(out.float().cpu().numpy(), O) <= TOL["bf16"]


def test_the_library_reports_which_kernels_a_call_would_run(torch, dsmoe):
    cfg = gen.CONFIGS["c3"]
    layer = dsmoe.Layer(cfg.d, cfg.f, cfg.E, "bf16", max_tokens=4096)
    path = lambda T, mode, k, eps: dsmoe.sparse_fwd_path(layer, T, mode, k, eps)
    assert path(1, dsmoe.SEL_TOPK, 4, 0.0) == dsmoe.PATH_FEW_TOKENS
    assert path(4, dsmoe.SEL_THRESHOLD, 0, 0.02) == dsmoe.PATH_FEW_TOKENS
    assert path(4, dsmoe.SEL_THRESHOLD_TOPK, 0, 0.02) == dsmoe.PATH_STREAMING     # the few-token kernels route themselves
    assert path(8, dsmoe.SEL_TOPK, 4, 0.0) == dsmoe.PATH_STREAMING
    assert path(8, dsmoe.SEL_THRESHOLD, 0, 0.02) == dsmoe.PATH_ALL_EXPERTS
    assert path(8, dsmoe.SEL_THRESHOLD | dsmoe.SEL_NORMALISED, 0, 0.64) == dsmoe.PATH_ALL_EXPERTS
    assert path(32, dsmoe.SEL_TOPK, 4, 0.0) == dsmoe.PATH_ALL_EXPERTS
    assert path(64, dsmoe.SEL_TOPK, 1, 0.0) == dsmoe.PATH_STREAMING               # too many experts stay idle
    assert path(128, dsmoe.SEL_TOPK, 4, 0.0) == dsmoe.PATH_STREAMING
    assert path(129, dsmoe.SEL_TOPK, 4, 0.0) == dsmoe.PATH_GROUPED
    assert path(0, dsmoe.SEL_TOPK, 4, 0.0) == dsmoe.PATH_GROUPED
    assert path(5000, dsmoe.SEL_TOPK, 4, 0.0) == -1 and path(8, 77, 4, 0.0) == -1
    f32 = dsmoe.Layer(256, 64, 8, "f32", max_tokens=64)
    assert dsmoe.sparse_fwd_path(f32, 1, dsmoe.SEL_TOPK, 2, 0.0) == dsmoe.PATH_GROUPED


@pytest.mark.parametrize("T,d,E,f,mode,k,eps,expert", [
    (48, 512, 64, 128, "topk", 8, 0.0, "swiglu"),          # 64 experts: eight per XCD, the six-stage variant
    (16, 320, 16, 192, "threshold", 0, 0.02, "swiglu"),    # ragged column slices in both phases
    (64, 256, 8, 64, "topk", 4, 0.0, "swiglu"),            # one expert per XCD, one slice per expert
    (24, 1024, 32, 256, "topk", 6, 0.0, "gelu"),
    (9, 2048, 32, 512, "threshold", 0, 0.01, "swiglu"),
])
def test_all_expert_decode_kernel_shapes(torch, dsmoe, T, d, E, f, mode, k, eps, expert):
    cfg = gen.LayerConfig("dense_decode", 25, T=T, d=d, E=E, f=f, dtype="bf16", mode=mode, k=k, eps=eps,
                          router_std=1.5 / np.sqrt(d))
    inp = conditioned(cfg, mode, k, eps, variant=T)
    if expert == "gelu":
        inp.w_up = None
    say(f"[case] all-expert decode kernel T={T} d={d} E={E} f={f} {mode} k={k} eps={eps} {expert}")
    w = weights_to_dev(torch, inp)
    layer = dsmoe.Layer(d, f, E, "bf16", max_tokens=T, expert=expert)
    code = mode_code(dsmoe, mode)
    assert dsmoe.sparse_fwd_path(layer, T, code, k, eps) == dsmoe.PATH_ALL_EXPERTS
    args = (w["x"], w["w_r"], w["b_r"], w["w_gate"], w["w_up"], w["w_down"], code, k, eps)
    out = layer.sparse_fwd(*args).clone()
    assert layer.poll_error() == dsmoe.OK
    probs, mask, eo, rt = layer.sparse_fwd_routing(T)
    torch.cuda.synchronize()
    O_ref, S_ref, M_ref = orc.sparse_forward(inp.x, inp.w_r, inp.b_r, inp.w_gate, inp.w_up, inp.w_down, mode, k, eps)
    assert helpers.rel_err(probs.cpu().numpy(), S_ref) <= 1e-5
    np.testing.assert_array_equal(mask_to_bool(mask, E), M_ref)
    r_ref = orc.dispatch(M_ref, S_ref)
    np.testing.assert_array_equal(eo.cpu().numpy(), r_ref.expert_off)
    np.testing.assert_array_equal(rt.cpu().numpy()[:r_ref.nnz], r_ref.row_token)
    err = helpers.rel_err(out.float().cpu().numpy(), O_ref)
    say(f"  rel err {err:.3e}")
    assert err <= TOL["bf16"]
    for _ in range(3):
        assert torch.equal(layer.sparse_fwd(*args), out)
    assert layer.poll_error() == dsmoe.OK
