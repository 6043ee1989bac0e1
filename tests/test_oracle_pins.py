"""Pins for the CPU checker (`oracle/dsmoe_oracle.py`): none of these re-use its formulas.

 * scalar brute force with `math` loops on tiny inputs (Eq. 1, selection, dispatch order);
 * a hand-sized layer whose router logits are exact rationals;
 * closed forms and invariants (K=E and eps=0 give the dense layer, one-hot router, permutations);
 * every gradient against central finite differences and against torch fp64 autograd of an
   independently written dense layer (Eq. 3 + chain rule).
"""
import math
import os

import numpy as np
import pytest

from oracle import dsmoe_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


# ------------------------------------------------------------------------------------------------
# independent scalar implementation (pure python floats)
# ------------------------------------------------------------------------------------------------
def s_silu(g):
    return g / (1.0 + math.exp(-g))


def s_softmax(z):
    m = max(z)
    ez = [math.exp(v - m) for v in z]
    s = sum(ez)
    return [v / s for v in ez]


def s_expert(x, wg, wu, wd):
    d, f = len(wg), len(wg[0])
    h = []
    for c in range(f):
        g = sum(x[i] * wg[i][c] for i in range(d))
        u = sum(x[i] * wu[i][c] for i in range(d))
        h.append(s_silu(g) * u)
    dout = len(wd[0])
    return [sum(h[c] * wd[c][k] for c in range(f)) for k in range(dout)]


def s_scores(x, w_r, b_r):
    E = len(w_r[0])
    z = [sum(x[i] * w_r[i][e] for i in range(len(x))) + (b_r[e] if b_r is not None else 0.0)
         for e in range(E)]
    return s_softmax(z)


def s_select(s, mode, k, eps):
    E = len(s)
    if mode == "topk":
        return sorted(sorted(range(E), key=lambda e: (-s[e], e))[:k])
    A = [e for e in range(E) if s[e] > eps]
    if not A:
        best = 0
        for e in range(1, E):
            if s[e] > s[best]:
                best = e
        A = [best]
    return A


def s_layer(X, w_r, b_r, wg, wu, wd, mode, k, eps):
    O, sets, scores = [], [], []
    for x in X:
        s = s_scores(x, w_r, b_r)
        A = s_select(s, mode, k, eps)
        o = [0.0] * len(wd[0][0])
        for e in A:
            y = s_expert(x, wg[e], wu[e], wd[e])
            o = [a + s[e] * b for a, b in zip(o, y)]
        O.append(o)
        sets.append(A)
        scores.append(s)
    return O, sets, scores


def rand_layer(seed, T, d, E, f, router_scale=1.0, bias=False):
    g = np.random.default_rng(seed)
    X = g.standard_normal((T, d))
    w_r = g.standard_normal((d, E)) * router_scale
    b_r = g.standard_normal(E) if bias else None
    wg = g.standard_normal((E, d, f)) * 0.5
    wu = g.standard_normal((E, d, f)) * 0.5
    wd = g.standard_normal((E, f, d)) * 0.5
    return X, w_r, b_r, wg, wu, wd


def load_tiny():
    out, name, shape, vals = {}, None, None, []
    with open(os.path.join(HERE, "golden", "tiny_layer.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0][0].isalpha():
                if name:
                    out[name] = np.array(vals, dtype=np.float64).reshape(shape)
                name, shape, vals = tok[0], tuple(int(v) for v in tok[1:]), []
            else:
                vals.extend(float(v) for v in tok)
    out[name] = np.array(vals, dtype=np.float64).reshape(shape)
    return out


# ------------------------------------------------------------------------------------------------
# hand-sized layer
# ------------------------------------------------------------------------------------------------
def test_tiny_layer_logits_are_the_hand_values():
    t = load_tiny()
    Z = orc.router_logits(t["X"], t["W_r"])
    np.testing.assert_allclose(Z, t["logits"], rtol=0, atol=1e-15)
    S = orc.softmax_rows(Z)
    den0 = 1.0 + math.exp(-1.25) + math.exp(0.25)
    np.testing.assert_allclose(S[0], [1.0 / den0, math.exp(-1.25) / den0, math.exp(0.25) / den0], rtol=1e-14)


@pytest.mark.parametrize("mode,k,eps,sets", [
    ("topk", 2, 0.0, [[0, 2], [0, 1]]),
    ("threshold", 0, 0.3, [[0, 2], [0]]),
    ("topk", 3, 0.0, [[0, 1, 2], [0, 1, 2]]),
])
def test_tiny_layer_against_scalar_code(mode, k, eps, sets):
    t = load_tiny()
    args = (t["X"], t["W_r"], None, t["W_gate"], t["W_up"], t["W_down"])
    O, S, M = orc.sparse_forward(*args, mode=mode, k=k, eps=eps)
    O_s, sets_s, S_s = s_layer(t["X"].tolist(), t["W_r"].tolist(), None, t["W_gate"].tolist(),
                               t["W_up"].tolist(), t["W_down"].tolist(), mode, k, eps)
    assert sets_s == sets                                   # the sets one reads off the logits by hand
    assert [list(np.nonzero(m)[0]) for m in M] == sets
    np.testing.assert_allclose(S, S_s, rtol=1e-14)
    np.testing.assert_allclose(O, O_s, rtol=1e-13, atol=1e-15)


def test_tiny_layer_dispatch_objects():
    t = load_tiny()
    S = orc.route(t["X"], t["W_r"])
    r = orc.dispatch(orc.select_topk(S, 2), S)
    assert r.cnt_exp.tolist() == [2, 1, 1]
    assert r.expert_off.tolist() == [0, 2, 3, 4]
    assert r.row_token.tolist() == [0, 1, 1, 0]
    assert r.tok_off.tolist() == [0, 2, 4]
    assert r.tok_rows.tolist() == [0, 3, 1, 2]
    assert r.mask_bits.tolist() == [0b101, 0b011]
    np.testing.assert_allclose(r.row_weight, [S[0, 0], S[1, 0], S[1, 1], S[0, 2]])


# ------------------------------------------------------------------------------------------------
# scalar brute force on random small layers
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("mode,k,eps", [("topk", 1, 0), ("topk", 3, 0), ("threshold", 0, 0.15),
                                        ("threshold", 0, 0.6)])
def test_sparse_forward_against_scalar_code(seed, mode, k, eps):
    X, w_r, b_r, wg, wu, wd = rand_layer(seed, T=7, d=4, E=5, f=3, bias=(seed == 1))
    O, S, M = orc.sparse_forward(X, w_r, b_r, wg, wu, wd, mode=mode, k=k, eps=eps)
    O_s, sets_s, S_s = s_layer(X.tolist(), w_r.tolist(), None if b_r is None else b_r.tolist(),
                               wg.tolist(), wu.tolist(), wd.tolist(), mode, k, eps)
    assert [list(np.nonzero(m)[0]) for m in M] == sets_s
    np.testing.assert_allclose(S, S_s, rtol=1e-13)
    np.testing.assert_allclose(O, O_s, rtol=1e-12, atol=1e-14)


def test_dispatch_against_nested_loops():
    g = np.random.default_rng(5)
    T, E = 37, 11
    M = g.random((T, E)) < 0.3
    M[np.arange(T), g.integers(0, E, T)] = True
    S = g.random((T, E))
    r = orc.dispatch(M, S)
    rows, row_of = [], {}
    for e in range(E):
        for t in range(T):
            if M[t, e]:
                row_of[(t, e)] = len(rows)
                rows.append((t, e))
    assert r.nnz == len(rows)
    assert r.row_token.tolist() == [t for t, _ in rows]
    np.testing.assert_array_equal(r.row_weight, [S[t, e] for t, e in rows])
    assert r.expert_off.tolist() == [sum(1 for _, e2 in rows if e2 < e) for e in range(E + 1)]
    tr = [row_of[(t, e)] for t in range(T) for e in range(E) if M[t, e]]
    assert r.tok_rows.tolist() == tr
    assert r.cnt_tok.tolist() == [int(M[t].sum()) for t in range(T)]
    assert [int(b) for b in r.mask_bits] == [sum(1 << e for e in range(E) if M[t, e]) for t in range(T)]
    # structural invariants
    assert r.cnt_tok.sum() == r.cnt_exp.sum() == r.expert_off[E] == r.tok_off[T] == r.nnz
    for e in range(E):
        seg = r.row_token[r.expert_off[e]:r.expert_off[e + 1]]
        assert np.all(np.diff(seg) > 0)
    assert sorted(r.tok_rows.tolist()) == list(range(r.nnz))


def test_staged_path_equals_fused_definition():
    X, w_r, b_r, wg, wu, wd = rand_layer(11, T=9, d=6, E=6, f=4)
    O, S, M = orc.sparse_forward(X, w_r, b_r, wg, wu, wd, mode="topk", k=3)
    r = orc.dispatch(M, S)
    Y = orc.expert_outputs_permuted(X, r, wg, wu, wd)
    np.testing.assert_allclose(orc.combine(Y, r, X.shape[0]), O, rtol=1e-13, atol=1e-15)


def test_token_subset_matches_full():
    X, w_r, b_r, wg, wu, wd = rand_layer(12, T=10, d=6, E=6, f=4)
    O, _, _ = orc.sparse_forward(X, w_r, b_r, wg, wu, wd, mode="threshold", eps=0.1)
    Os, _, _ = orc.sparse_forward(X, w_r, b_r, wg, wu, wd, mode="threshold", eps=0.1, tokens=[7, 2, 2])
    np.testing.assert_allclose(Os, O[[7, 2, 2]], rtol=1e-13, atol=1e-15)
    D, _, Yd = orc.dense_forward(X, w_r, b_r, wg, wu, wd)
    Ds, _, _ = orc.dense_forward(X, w_r, b_r, wg, wu, wd, tokens=[3, 9])
    np.testing.assert_allclose(Ds, D[[3, 9]], rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------------------------------------------
# selection rules, ties, fallback
# ------------------------------------------------------------------------------------------------
def test_topk_ties_go_to_lower_index():
    S = np.array([[0.2, 0.3, 0.3, 0.2], [0.25, 0.25, 0.25, 0.25]])
    assert orc.select_topk(S, 1).tolist() == [[False, True, False, False], [True, False, False, False]]
    assert orc.select_topk(S, 3).tolist() == [[True, True, True, False], [True, True, True, False]]


def test_duplicated_router_columns_tie_exactly():
    X, w_r, _, wg, wu, wd = rand_layer(3, T=16, d=8, E=4, f=3)
    w_r[:, 2] = w_r[:, 0]                     # bit-identical logits for experts 0 and 2
    S = orc.route(X, w_r)
    assert np.array_equal(S[:, 0], S[:, 2])
    M = orc.select_topk(S, 1)
    assert not M[:, 2].any()                  # expert 2 can never beat its lower-index twin
    M3 = orc.select_topk(S, 3)
    assert np.all(M3[:, 0] | ~M3[:, 2])


def test_threshold_is_strict_and_falls_back_to_argmax():
    S = np.array([[0.5, 0.3, 0.2], [0.2, 0.4, 0.4], [0.1, 0.1, 0.8]])
    assert orc.select_threshold(S, 0.3).tolist() == [[True, False, False], [False, True, True],
                                                     [False, False, True]]
    assert orc.select_threshold(S, 0.9).tolist() == [[True, False, False], [False, True, False],
                                                     [False, False, True]]


def test_threshold_topk_average():
    S = np.array([[0.5, 0.3, 0.2], [0.2, 0.4, 0.4], [0.1, 0.1, 0.8], [0.34, 0.33, 0.33]])
    # above 0.25: 2, 2, 1, 3 experts -> mean 2.0
    assert orc.threshold_topk_k(S, 0.25) == 2
    # above 0.35: 1, 2, 1, 0 (-> argmax fallback 1) -> mean 1.25 -> 1
    assert orc.threshold_topk_k(S, 0.35) == 1


# ------------------------------------------------------------------------------------------------
# invariants and closed forms
# ------------------------------------------------------------------------------------------------
def wide_swiglu_dense(X, w_r, b_r, wg, wu, wd):
    """Dense layer written as ONE SwiGLU block of width E*f with the hidden blocks scaled by S."""
    T, d = X.shape
    E, _, f = wg.shape
    z = X @ w_r + (0 if b_r is None else b_r)
    z = z - z.max(axis=1, keepdims=True)
    S = np.exp(z) / np.exp(z).sum(axis=1, keepdims=True)
    Wg = np.concatenate(list(wg), axis=1)
    Wu = np.concatenate(list(wu), axis=1)
    Wd = np.concatenate(list(wd), axis=0)
    G = X @ Wg
    H = (G / (1 + np.exp(-G))) * (X @ Wu) * np.repeat(S, f, axis=1)
    return H @ Wd


def test_dense_forward_is_one_wide_swiglu():
    X, w_r, b_r, wg, wu, wd = rand_layer(21, T=13, d=8, E=5, f=4, bias=True)
    O, S, Y = orc.dense_forward(X, w_r, b_r, wg, wu, wd)
    np.testing.assert_allclose(O, wide_swiglu_dense(X, w_r, b_r, wg, wu, wd), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(S.sum(axis=1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(np.einsum("te,ted->td", S, Y), O, rtol=1e-13)


def test_k_equals_E_and_eps_zero_give_the_dense_layer():
    X, w_r, b_r, wg, wu, wd = rand_layer(22, T=11, d=8, E=6, f=4)
    D, _, _ = orc.dense_forward(X, w_r, b_r, wg, wu, wd)
    O1, _, M1 = orc.sparse_forward(X, w_r, b_r, wg, wu, wd, mode="topk", k=6)
    O2, _, M2 = orc.sparse_forward(X, w_r, b_r, wg, wu, wd, mode="threshold", eps=0.0)
    assert M1.all() and M2.all()
    np.testing.assert_allclose(O1, D, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(O2, D, rtol=1e-13, atol=1e-15)


def test_one_hot_router_reproduces_a_single_expert():
    X, w_r, _, wg, wu, wd = rand_layer(23, T=6, d=8, E=4, f=5)
    w_r[:] = 0.0
    b_r = np.array([0.0, 0.0, 800.0, 0.0])
    for mode, k, eps in (("topk", 1, 0), ("threshold", 0, 0.5), ("topk", 4, 0)):
        O, S, M = orc.sparse_forward(X, w_r, b_r, wg, wu, wd, mode=mode, k=k, eps=eps)
        np.testing.assert_array_equal(S[:, 2], 1.0)
        single = np.array(s_layer(X.tolist(), w_r.tolist(), b_r.tolist(), wg.tolist(), wu.tolist(),
                                  wd.tolist(), "topk", 1, 0)[0])
        np.testing.assert_allclose(O, single, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(O, [s_expert(x, wg[2].tolist(), wu[2].tolist(), wd[2].tolist())
                                       for x in X.tolist()], rtol=1e-12, atol=1e-14)


def test_top1_is_the_argmax_expert():
    X, w_r, b_r, wg, wu, wd = rand_layer(24, T=9, d=8, E=5, f=3)
    O, S, M = orc.sparse_forward(X, w_r, b_r, wg, wu, wd, mode="topk", k=1)
    for t in range(X.shape[0]):
        e = int(np.argmax(S[t]))
        assert M[t].tolist() == [j == e for j in range(5)]
        y = s_expert(X[t].tolist(), wg[e].tolist(), wu[e].tolist(), wd[e].tolist())
        np.testing.assert_allclose(O[t], S[t, e] * np.array(y), rtol=1e-13)


def test_zero_router_gives_uniform_scores_and_mean_of_experts():
    X, w_r, _, wg, wu, wd = rand_layer(25, T=5, d=6, E=4, f=3)
    w_r[:] = 0.0
    O, S, _ = orc.dense_forward(X, w_r, None, wg, wu, wd)
    np.testing.assert_array_equal(S, 0.25)
    mean = np.mean([[s_expert(x, wg[e].tolist(), wu[e].tolist(), wd[e].tolist()) for e in range(4)]
                    for x in X.tolist()], axis=1)
    np.testing.assert_allclose(O, mean, rtol=1e-13)
    # eps >= 1/E: nothing exceeds it, every token falls back to expert 0
    _, _, M = orc.sparse_forward(X, w_r, None, wg, wu, wd, mode="threshold", eps=0.25)
    assert M[:, 0].all() and not M[:, 1:].any()


def test_zero_gate_gives_zero_output():
    X, w_r, b_r, wg, wu, wd = rand_layer(26, T=5, d=6, E=4, f=3)
    O, _, _ = orc.dense_forward(X, w_r, b_r, np.zeros_like(wg), wu, wd)
    np.testing.assert_array_equal(O, 0.0)


def test_token_and_expert_permutations():
    X, w_r, b_r, wg, wu, wd = rand_layer(27, T=12, d=8, E=6, f=4, bias=True)
    O, S, M = orc.sparse_forward(X, w_r, b_r, wg, wu, wd, mode="topk", k=2)
    g = np.random.default_rng(0)
    pt = g.permutation(12)
    Op, Sp, Mp = orc.sparse_forward(X[pt], w_r, b_r, wg, wu, wd, mode="topk", k=2)
    np.testing.assert_array_equal(Op, O[pt])
    assert orc.dispatch(Mp, Sp).cnt_exp.tolist() == orc.dispatch(M, S).cnt_exp.tolist()
    pe = g.permutation(6)
    Oe, Se, Me = orc.sparse_forward(X, w_r[:, pe], b_r[pe], wg[pe], wu[pe], wd[pe], mode="topk", k=2)
    np.testing.assert_allclose(Oe, O, rtol=1e-12, atol=1e-14)
    assert orc.dispatch(Me, Se).cnt_exp.tolist() == orc.dispatch(M, S).cnt_exp[pe].tolist()


# ------------------------------------------------------------------------------------------------
# gradients (Eq. 3 + chain rule)
# ------------------------------------------------------------------------------------------------
def loss_fn(X, w_r, b_r, wg, wu, wd, dO):
    return float((wide_swiglu_dense(X, w_r, b_r, wg, wu, wd) * dO).sum())


@pytest.mark.parametrize("bias", [False, True])
def test_dense_backward_against_finite_differences(bias):
    X, w_r, b_r, wg, wu, wd = rand_layer(31, T=4, d=3, E=3, f=2, bias=bias)
    dO = np.random.default_rng(9).standard_normal(X.shape)
    gr = orc.dense_backward(X, w_r, b_r, wg, wu, wd, dO)
    params = {"X": (X, gr.dX), "w_r": (w_r, gr.dW_r), "wg": (wg, gr.dW_gate), "wu": (wu, gr.dW_up),
              "wd": (wd, gr.dW_down)}
    if bias:
        params["b_r"] = (b_r, gr.db_r)
    h = 1e-6
    for name, (p, g_an) in params.items():
        g_fd = np.zeros_like(p)
        it = np.nditer(p, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = p[idx]
            p[idx] = old + h
            lp = loss_fn(X, w_r, b_r, wg, wu, wd, dO)
            p[idx] = old - h
            lm = loss_fn(X, w_r, b_r, wg, wu, wd, dO)
            p[idx] = old
            g_fd[idx] = (lp - lm) / (2 * h)
        np.testing.assert_allclose(g_an, g_fd, rtol=2e-6, atol=2e-8, err_msg=name)


def test_dense_backward_against_torch_autograd():
    torch = pytest.importorskip("torch")
    X, w_r, b_r, wg, wu, wd = rand_layer(32, T=24, d=16, E=6, f=8, bias=True)
    dO = np.random.default_rng(10).standard_normal(X.shape)
    tt = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True)
          for k, v in dict(X=X, w_r=w_r, b_r=b_r, wg=wg, wu=wu, wd=wd).items()}
    S = torch.softmax(tt["X"] @ tt["w_r"] + tt["b_r"], dim=1)
    G = torch.einsum("td,edf->tef", tt["X"], tt["wg"])
    U = torch.einsum("td,edf->tef", tt["X"], tt["wu"])
    Y = torch.einsum("tef,efd->ted", torch.nn.functional.silu(G) * U, tt["wd"])
    Y.retain_grad()
    S.retain_grad()
    O = (S[:, :, None] * Y).sum(dim=1)
    O.backward(torch.tensor(dO))
    gr = orc.dense_backward(X, w_r, b_r, wg, wu, wd, dO)
    O_or, S_or, Y_or = orc.dense_forward(X, w_r, b_r, wg, wu, wd)
    np.testing.assert_allclose(O_or, O.detach().numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(Y_or, Y.detach().numpy(), rtol=1e-12, atol=1e-14)
    for got, name in ((gr.dX, "X"), (gr.dW_r, "w_r"), (gr.db_r, "b_r"), (gr.dW_gate, "wg"),
                      (gr.dW_up, "wu"), (gr.dW_down, "wd")):
        np.testing.assert_allclose(got, tt[name].grad.numpy(), rtol=1e-11, atol=1e-13, err_msg=name)
    # Eq. 3 literally: grad S = [e_1(X) .. e_N(X)]^T grad O,  grad e_j(X) = S_j grad O
    np.testing.assert_allclose(gr.dS, S.grad.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(Y.grad.numpy(), S_or[:, :, None] * dO[:, None, :], rtol=1e-13)
    np.testing.assert_allclose(gr.dZ.sum(axis=1), 0.0, atol=1e-12)


def test_expert_backward_sums_to_the_layer_backward():
    X, w_r, b_r, wg, wu, wd = rand_layer(33, T=6, d=5, E=4, f=3)
    dO = np.random.default_rng(11).standard_normal(X.shape)
    gr = orc.dense_backward(X, w_r, b_r, wg, wu, wd, dO)
    S = orc.route(X, w_r, b_r)
    dX = gr.dZ @ w_r.T
    for j in range(4):
        dxj, dwg, dwu, dwd = orc.expert_backward(X, S[:, j], wg[j], wu[j], wd[j], dO)
        dX = dX + dxj
        np.testing.assert_array_equal(dwd, gr.dW_down[j])
        np.testing.assert_array_equal(dwg, gr.dW_gate[j])
    np.testing.assert_allclose(dX, gr.dX, rtol=1e-13)


# ------------------------------------------------------------------------------------------------
# mutual-information loss (Eq. 4-5): closed forms and finite differences
# ------------------------------------------------------------------------------------------------
def test_mi_loss_closed_forms():
    E = 8
    assert abs(orc.mi_loss(np.full((5, E), 1.0 / E))) < 1e-15            # -ln E + ln E
    onehot = np.eye(E)[np.arange(16) % E]
    assert abs(orc.mi_loss(onehot) + math.log(E)) < 1e-15                # balanced one-hot: -ln E
    collapsed = np.eye(E)[np.zeros(16, dtype=int)]
    assert abs(orc.mi_loss(collapsed)) < 1e-15                           # all on one expert: 0 + 0


def test_mi_loss_grad_against_finite_differences():
    g = np.random.default_rng(4)
    S = g.random((5, 4)) + 0.1
    S /= S.sum(axis=1, keepdims=True)
    an = orc.mi_loss_grad(S)
    h = 1e-7
    for idx in np.ndindex(*S.shape):
        Sp, Sm = S.copy(), S.copy()
        Sp[idx] += h
        Sm[idx] -= h
        assert abs((orc.mi_loss(Sp) - orc.mi_loss(Sm)) / (2 * h) - an[idx]) < 1e-6


def test_mi_backward_against_finite_differences_of_the_router():
    # alpha * L_MI as a function of the router's parameters and input, differentiated numerically
    g = np.random.default_rng(21)
    T, d, E, alpha = 6, 5, 4, 0.7
    X, w_r, b_r = g.standard_normal((T, d)), 0.5 * g.standard_normal((d, E)), 0.3 * g.standard_normal(E)
    loss = lambda X_, w_, b_: alpha * orc.mi_loss(orc.route(X_, w_, b_))
    dX, dW, db = orc.mi_backward(X, w_r, b_r, alpha)
    h = 1e-6
    for arr, grad, pos in ((X, dX, 0), (w_r, dW, 1), (b_r, db, 2)):
        for idx in np.ndindex(*arr.shape):
            args_p, args_m = [X.copy(), w_r.copy(), b_r.copy()], [X.copy(), w_r.copy(), b_r.copy()]
            args_p[pos][idx] += h
            args_m[pos][idx] -= h
            num = (loss(*args_p) - loss(*args_m)) / (2 * h)
            assert abs(num - grad[idx]) < 1e-7, (pos, idx, num, grad[idx])


def test_mi_backward_vanishes_for_a_constant_router():
    # W_r = 0: every token has the same scores, p = S, so log p - log S = 0 and nothing flows back
    X = np.random.default_rng(3).standard_normal((7, 5))
    dX, dW, db = orc.mi_backward(X, np.zeros((5, 4)), np.array([0.3, -0.2, 0.0, 0.1]), 1.0)
    assert np.abs(dX).max() < 1e-15 and np.abs(dW).max() < 1e-15 and np.abs(db).max() < 1e-15


def test_threshold_topk_selection_is_topk_at_the_batch_mean_count():
    # hand case: counts above 0.25 are (2, 1, 3) -> mean 2 -> top-2 of every token
    S = np.array([[0.40, 0.30, 0.20, 0.10],
                  [0.70, 0.10, 0.10, 0.10],
                  [0.30, 0.28, 0.26, 0.16]])
    M = orc.select_threshold_topk(S, 0.25)
    np.testing.assert_array_equal(M, np.array([[1, 1, 0, 0], [1, 1, 0, 0], [1, 1, 0, 0]], dtype=bool))
    # rounding half up: counts (1, 2) -> mean 1.5 -> K = 2
    S2 = np.array([[0.60, 0.20, 0.15, 0.05], [0.45, 0.40, 0.10, 0.05]])
    assert orc.threshold_topk_k(S2, 0.25) == 2
    assert orc.select_threshold_topk(S2, 0.25).sum(axis=1).tolist() == [2, 2]


# ------------------------------------------------------------------------------------------------
# the paper's own expert: two matrices and GeLU (Sec. 4.1); selected by passing W_up = None
# ------------------------------------------------------------------------------------------------
def s_gelu(g):
    return 0.5 * g * (1.0 + math.erf(g / math.sqrt(2.0)))


def s_expert_gelu(x, w1, w2):
    d, f = len(w1), len(w1[0])
    h = [s_gelu(sum(x[i] * w1[i][c] for i in range(d))) for c in range(f)]
    return [sum(h[c] * w2[c][k] for c in range(f)) for k in range(len(w2[0]))]


def test_gelu_known_values_and_identities():
    # Phi(1) and Phi(2) from any table of the standard normal CDF
    assert abs(orc.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15
    assert abs(orc.gelu(np.array([2.0]))[0] - 2 * 0.9772498680518208) < 1e-15
    g = np.linspace(-6, 6, 241)
    # Phi(g) + Phi(-g) = 1  =>  gelu(g) - gelu(-g) = g
    np.testing.assert_allclose(orc.gelu(g) - orc.gelu(-g), g, rtol=0, atol=1e-15)
    assert orc.gelu(np.array([0.0]))[0] == 0.0
    assert abs(orc.gelu(np.array([30.0]))[0] - 30.0) < 1e-12 and abs(orc.gelu(np.array([-30.0]))[0]) < 1e-12
    # derivative by central differences
    h = 1e-6
    np.testing.assert_allclose(orc.gelu_prime(g), (orc.gelu(g + h) - orc.gelu(g - h)) / (2 * h), atol=1e-9)


@pytest.mark.parametrize("mode,k,eps", [("topk", 2, 0), ("threshold", 0, 0.2)])
def test_gelu_expert_sparse_forward_against_scalar_code(mode, k, eps):
    X, w_r, b_r, w1, _, w2 = rand_layer(41, T=7, d=5, E=4, f=3, bias=True)
    O, S, M = orc.sparse_forward(X, w_r, b_r, w1, None, w2, mode, k, eps)
    for t in range(X.shape[0]):
        s = s_scores(X[t].tolist(), w_r.tolist(), b_r.tolist())
        A = s_select(s, mode, k, eps)
        assert np.nonzero(M[t])[0].tolist() == A
        o = np.zeros(X.shape[1])
        for e in A:
            o += s[e] * np.array(s_expert_gelu(X[t].tolist(), w1[e].tolist(), w2[e].tolist()))
        np.testing.assert_allclose(O[t], o, rtol=1e-12, atol=1e-14)
    # staged path (dispatch, per-expert rows, combine) equals the fused definition
    r = orc.dispatch(M, S)
    Y = orc.expert_outputs_permuted(X, r, w1, None, w2)
    np.testing.assert_allclose(orc.combine(Y, r, X.shape[0]), O, rtol=1e-12, atol=1e-14)


def test_gelu_expert_dense_backward_against_torch_autograd_and_finite_differences():
    torch = pytest.importorskip("torch")
    X, w_r, b_r, w1, _, w2 = rand_layer(42, T=10, d=6, E=4, f=5, bias=True)
    dO = np.random.default_rng(12).standard_normal(X.shape)
    tt = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True)
          for k, v in dict(X=X, w_r=w_r, b_r=b_r, w1=w1, w2=w2).items()}
    S = torch.softmax(tt["X"] @ tt["w_r"] + tt["b_r"], dim=1)
    G = torch.einsum("td,edf->tef", tt["X"], tt["w1"])
    Y = torch.einsum("tef,efd->ted", torch.nn.functional.gelu(G), tt["w2"])     # exact (erf) GeLU
    O = (S[:, :, None] * Y).sum(dim=1)
    O.backward(torch.tensor(dO))
    gr = orc.dense_backward(X, w_r, b_r, w1, None, w2, dO)
    O_or, _, _ = orc.dense_forward(X, w_r, b_r, w1, None, w2)
    np.testing.assert_allclose(O_or, O.detach().numpy(), rtol=1e-12, atol=1e-14)
    assert gr.dW_up is None
    for got, name in ((gr.dX, "X"), (gr.dW_r, "w_r"), (gr.db_r, "b_r"), (gr.dW_gate, "w1"), (gr.dW_down, "w2")):
        np.testing.assert_allclose(got, tt[name].grad.numpy(), rtol=1e-10, atol=1e-12, err_msg=name)
    # one entry of each gradient by central differences of the scalar loss <O, dO>
    loss = lambda: float((orc.dense_forward(X, w_r, b_r, w1, None, w2)[0] * dO).sum())
    h = 1e-6
    for p, g_an, idx in ((X, gr.dX, (3, 2)), (w1, gr.dW_gate, (1, 4, 2)), (w2, gr.dW_down, (2, 3, 1)),
                         (w_r, gr.dW_r, (5, 0))):
        old = p[idx]
        p[idx] = old + h
        lp = loss()
        p[idx] = old - h
        lm = loss()
        p[idx] = old
        assert abs((lp - lm) / (2 * h) - g_an[idx]) < 1e-6 * max(1.0, abs(g_an[idx]))
