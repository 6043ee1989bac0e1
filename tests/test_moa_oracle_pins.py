"""Pins of the MoA checker (oracle/moa_oracle.py) against things other than itself: scalar brute force,
scipy's softmax, closed forms and invariants of Eq. 7-8 (Sec. 3.2)."""
import math

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

import dsmoe_inputs as gen
from oracle import dsmoe_oracle as moe
from oracle import moa_oracle as moa


def tiny(T=5, L=7, d=6, E=4, n_head=2, d_head=3, seed=0):
    rng = np.random.default_rng(seed)
    hd = n_head * d_head
    return dict(X=rng.standard_normal((T, d)), W_r=rng.standard_normal((d, E)), b_r=rng.standard_normal(E),
                W_q=rng.standard_normal((E, d, hd)), K=rng.standard_normal((n_head, L, d_head)),
                V=rng.standard_normal((n_head, L, d_head)), W_o=rng.standard_normal((E, hd, d)))


def brute_force(p, selected, scale):
    """Eq. 7-8 with Python scalars only: selected[t] lists the experts of token t."""
    X, W_r, b_r, W_q, K, V, W_o = (p[k] for k in ("X", "W_r", "b_r", "W_q", "K", "V", "W_o"))
    T, d = X.shape
    E, n_head, L, d_head = W_q.shape[0], K.shape[0], K.shape[1], K.shape[2]
    O = [[0.0] * d for _ in range(T)]
    for t in range(T):
        z = [sum(X[t][a] * W_r[a][e] for a in range(d)) + b_r[e] for e in range(E)]
        zmax = max(z)
        ez = [math.exp(v - zmax) for v in z]
        S = [v / sum(ez) for v in ez]
        last = L - T + t
        for i in selected[t]:
            for j in range(n_head):
                q = [sum(X[t][a] * W_q[i][a][j * d_head + c] for a in range(d)) for c in range(d_head)]
                a_l = [scale * sum(q[c] * K[j][l][c] for c in range(d_head)) for l in range(last + 1)]
                amax = max(a_l)
                ea = [math.exp(v - amax) for v in a_l]
                pl = [v / sum(ea) for v in ea]
                ctx = [sum(pl[l] * V[j][l][c] for l in range(last + 1)) for c in range(d_head)]
                for o in range(d):
                    O[t][o] += S[i] * sum(ctx[c] * W_o[i][j * d_head + c][o] for c in range(d_head))
    return np.array(O)


@pytest.mark.parametrize("scale", [1.0, 0.5])
def test_scalar_brute_force_topk(scale):
    p = tiny()
    O, S, M = moa.moa_forward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], "topk", k=2, scale=scale)
    # the selection itself is pinned with the MLP layer's checker; here the two highest scores, by hand
    selected = [sorted(np.argsort(-S[t], kind="stable")[:2]) for t in range(S.shape[0])]
    assert [list(np.nonzero(M[t])[0]) for t in range(M.shape[0])] == [list(s) for s in selected]
    np.testing.assert_allclose(O, brute_force(p, selected, scale), rtol=1e-11, atol=1e-12)


def test_dense_mode_is_brute_force_over_all_experts():
    p = tiny(seed=3)
    O, _, M = moa.moa_forward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], "dense", scale=0.7)
    assert M.all()
    np.testing.assert_allclose(O, brute_force(p, [range(4)] * 5, 0.7), rtol=1e-11, atol=1e-12)


def test_one_expert_one_head_is_textbook_causal_attention():
    """A router that always picks expert 2 with score ~1, one head: Eq. 7-8 reduce to causal softmax attention,
    written here with scipy's softmax and a triangular mask."""
    p = tiny(T=6, L=6, n_head=1, d_head=4, seed=5)
    p["W_r"] = np.zeros_like(p["W_r"])
    p["b_r"] = np.array([0.0, 0.0, 80.0, 0.0])
    O, S, _ = moa.moa_forward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], "topk", k=1, scale=0.5)
    Q = p["X"] @ p["W_q"][2]
    A = 0.5 * Q @ p["K"][0].T
    A[np.triu_indices(6, k=1)] = -np.inf
    ref = scipy_softmax(A, axis=1) @ p["V"][0] @ p["W_o"][2]
    np.testing.assert_allclose(O, ref, rtol=1e-10, atol=1e-12)


def test_constant_values_closed_form():
    """If every cached value of head j is the same vector v_j, attention returns v_j whatever Q and K are:
    O = sum_i S_i sum_j v_j W_o[i][j]."""
    p = tiny(seed=7)
    vj = np.random.default_rng(1).standard_normal((2, 3))
    p["V"] = np.repeat(vj[:, None, :], p["K"].shape[1], axis=1)
    O, S, _ = moa.moa_forward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], "dense", scale=1.3)
    per_expert = np.stack([vj.reshape(-1) @ p["W_o"][i] for i in range(4)])      # [E, d]
    np.testing.assert_allclose(O, S @ per_expert, rtol=1e-11, atol=1e-12)


def test_zero_scale_averages_the_visible_values():
    p = tiny(T=4, L=9, seed=9)
    O, S, _ = moa.moa_forward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], "dense", scale=0.0)
    T, L = 4, 9
    ref = np.zeros_like(O)
    for t in range(T):
        n = L - T + t + 1
        mean = p["V"][:, :n, :].mean(axis=1).reshape(-1)                          # [n_head * d_head]
        ref[t] = sum(S[t, i] * (mean @ p["W_o"][i]) for i in range(4))
    np.testing.assert_allclose(O, ref, rtol=1e-11, atol=1e-12)


def test_causality_and_cache_order():
    p = tiny(T=3, L=8, seed=11)
    args = lambda q: (q["X"], q["W_r"], q["b_r"], q["W_q"], q["K"], q["V"], q["W_o"], "topk")
    O, _, _ = moa.moa_forward(*args(p), k=2, scale=0.8)
    # positions after a token's own do not reach it: token 0 sits at position 5
    q = {k: v.copy() for k, v in p.items()}
    q["K"][:, 6:, :] += 3.0
    q["V"][:, 6:, :] -= 2.0
    O2, _, _ = moa.moa_forward(*args(q), k=2, scale=0.8)
    np.testing.assert_array_equal(O[0], O2[0])
    assert np.abs(O[2] - O2[2]).max() > 1e-3
    # the order of the positions every token sees (0..5) does not matter
    perm = np.array([3, 1, 5, 0, 4, 2, 6, 7])
    r = {k: v.copy() for k, v in p.items()}
    r["K"], r["V"] = p["K"][:, perm, :], p["V"][:, perm, :]
    O3, _, _ = moa.moa_forward(*args(r), k=2, scale=0.8)
    np.testing.assert_allclose(O3, O, rtol=1e-12, atol=1e-13)


def test_expert_order_and_k_equals_n():
    p = tiny(seed=13)
    O, _, _ = moa.moa_forward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], "topk", k=2, scale=1.0)
    perm = np.array([2, 0, 3, 1])
    Op, _, _ = moa.moa_forward(p["X"], p["W_r"][:, perm], p["b_r"][perm], p["W_q"][perm], p["K"], p["V"],
                               p["W_o"][perm], "topk", k=2, scale=1.0)
    np.testing.assert_allclose(Op, O, rtol=1e-12, atol=1e-13)
    Ok, _, _ = moa.moa_forward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], "topk", k=4, scale=1.0)
    Od, _, _ = moa.moa_forward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], "dense", scale=1.0)
    np.testing.assert_allclose(Ok, Od, rtol=1e-12, atol=1e-13)


def test_generator_shapes_follow_table_1():
    cfg = gen.MOA_CONFIGS["m2"]
    assert (cfg.d, cfg.E, cfg.n_head, cfg.d_head) == (4096, 8, 4, 128)          # DS-MoE-6B row
    inp = gen.make_moa(gen.MOA_CONFIGS["m1"])
    assert inp.w_q.shape == (8, 128, 128) and inp.k.shape == (2, 80, 64) and inp.w_o.shape == (8, 128, 128)
    again = gen.make_moa(gen.MOA_CONFIGS["m1"])
    np.testing.assert_array_equal(inp.k, again.k)


# ---- dense-training gradients of the attention layer ---------------------------------------------------
def _loss(p, dO, scale):
    O, _, _ = moa.moa_forward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], "dense", scale=scale)
    return float((O * dO).sum())


@pytest.mark.parametrize("scale", [1.0, 0.6])
def test_dense_backward_against_central_differences(scale):
    p = tiny(T=4, L=6, d=5, E=3, n_head=2, d_head=3, seed=21)
    dO = np.random.default_rng(2).standard_normal(p["X"].shape)
    g = moa.moa_dense_backward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], dO, scale)
    h = 1e-6
    for name, key in (("dX", "X"), ("dW_r", "W_r"), ("db_r", "b_r"), ("dW_q", "W_q"), ("dW_o", "W_o"), ("dK", "K"),
                      ("dV", "V")):
        num = np.zeros_like(p[key])
        it = np.nditer(p[key], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            keep = p[key][idx]
            p[key][idx] = keep + h
            up = _loss(p, dO, scale)
            p[key][idx] = keep - h
            dn = _loss(p, dO, scale)
            p[key][idx] = keep
            num[idx] = (up - dn) / (2 * h)
        np.testing.assert_allclose(g[name], num, rtol=2e-6, atol=2e-8, err_msg=name)


def test_dense_backward_against_autograd_of_an_independent_layer():
    torch = pytest.importorskip("torch")
    p = tiny(T=5, L=8, d=6, E=4, n_head=2, d_head=4, seed=23)
    dO = np.random.default_rng(4).standard_normal(p["X"].shape)
    scale = 0.5
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    T, L = 5, 8
    S = torch.softmax(t["X"] @ t["W_r"] + t["b_r"], dim=1)
    Q = torch.einsum("td,edh->eth", t["X"], t["W_q"]).reshape(4, T, 2, 4)              # [E, T, head, d_head]
    att = scale * torch.einsum("etjc,jlc->ejtl", Q, t["K"])                             # [E, head, T, L]
    visible = torch.arange(L)[None, :] <= (L - T + torch.arange(T))[:, None]
    att = att.masked_fill(~visible, float("-inf"))
    ctx = torch.einsum("ejtl,jlc->etjc", torch.softmax(att, dim=-1), t["V"]).reshape(4, T, 8)
    O = torch.einsum("te,eth,ehd->td", S, ctx, t["W_o"])
    (O * torch.tensor(dO)).sum().backward()
    g = moa.moa_dense_backward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], dO, scale)
    for name, key in (("dX", "X"), ("dW_r", "W_r"), ("db_r", "b_r"), ("dW_q", "W_q"), ("dW_o", "W_o"), ("dK", "K"),
                      ("dV", "V")):
        np.testing.assert_allclose(g[name], t[key].grad.numpy(), rtol=1e-10, atol=1e-12, err_msg=name)
    # and the forward of that layer is the checker's forward
    Oc, _, _ = moa.moa_forward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], "dense", scale=scale)
    np.testing.assert_allclose(Oc, O.detach().numpy(), rtol=1e-11, atol=1e-13)


def test_score_gradient_is_the_inner_product_of_eq_3():
    p = tiny(seed=25)
    dO = np.random.default_rng(6).standard_normal(p["X"].shape)
    g = moa.moa_dense_backward(p["X"], p["W_r"], p["b_r"], p["W_q"], p["K"], p["V"], p["W_o"], dO, 1.0)
    for i in range(4):
        e_i = moa.expert_heads(p["X"], p["W_q"][i], p["K"], p["V"], p["W_o"][i], p["K"].shape[1] - p["X"].shape[0], 1.0)
        np.testing.assert_allclose(g["dS"][:, i], (e_i * dO).sum(axis=1), rtol=1e-12, atol=1e-13)
