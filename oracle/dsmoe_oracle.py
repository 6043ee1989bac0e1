"""CPU checker for the DS-MoE expert layer: the layer's plain definition in fp64.

TEST INFRASTRUCTURE ONLY.  This file is the reference the GPU library is compared against.  It is
imported by the test-suite, by the smoke check and by the benchmark's CPU-baseline leg, and by nothing
else; the product never routes through it and it shares no code with the HIP path.

The method is exact (not an approximation), so every function below is the defining formula written
out with numpy fp64 array operations; `@` (a library matrix product) is the only library primitive
used for the contractions (and scipy's erf for the GeLU expert).  There is no blocking, fusion or reordering beyond what the formulas state.

Notation follows the paper (Sec. 3.1): a token X in R^{d_h}, N experts e_1..e_N, router scores
S = softmax(h(X)), selected index set A.  Array shapes: X[T,d], W_r[d,E], b_r[E], W_gate/W_up[E,d,f],
W_down[E,f,d]; T tokens, E = N experts.

Readings taken where the paper is silent (listed with reasons in the design notes):
  * the router h is one linear map X W_r (+ b_r);
  * an expert is a SwiGLU MLP, e(x) = (silu(x W_gate) * (x W_up)) W_down, without biases (the paper
    says only "MLP module" and uses GeLU; the workload definition fixes SwiGLU); passing W_up = None
    selects the paper's own two-matrix expert, e(x) = gelu(x W_1) W_2 with the exact (erf) GeLU;
  * the kept scores are used as they are (Eq. 1 has no renormalisation over the kept set);
  * the threshold is applied to the raw probability, strictly (S > eps); the paper's normalised
    threshold (Sec. 4.2 footnote: probability times N) is eps_raw = eps_paper / N;
  * ties in top-K and in the argmax fall to the lower expert index; a token with no score above the
    threshold keeps its argmax expert.

Every function here is pinned by tests that do not re-use it (scalar brute force, closed forms,
invariants, finite differences, an autograd cross-check); nothing is "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np
from scipy.special import erf as _erf   # library primitive for the GeLU expert only

F64 = np.float64


def _f64(a):
    return None if a is None else np.asarray(a, dtype=F64)


# --------------------------------------------------------------------------------------------------
# Router: Eq. 1, first half.
# --------------------------------------------------------------------------------------------------
def router_logits(X, W_r, b_r=None) -> np.ndarray:
    """h(X): one score per expert and token, Z[t,e] = sum_i X[t,i] W_r[i,e] (+ b_r[e])."""
    Z = _f64(X) @ _f64(W_r)
    if b_r is not None:
        Z = Z + _f64(b_r)[None, :]
    return Z


def softmax_rows(Z) -> np.ndarray:
    """S = softmax(Z) over all N experts of each token (Eq. 1), max-subtracted."""
    Z = _f64(Z)
    ez = np.exp(Z - Z.max(axis=1, keepdims=True))
    return ez / ez.sum(axis=1, keepdims=True)


def route(X, W_r, b_r=None) -> np.ndarray:
    """S[T,E] = softmax(h(X)) (Eq. 1)."""
    return softmax_rows(router_logits(X, W_r, b_r))


# --------------------------------------------------------------------------------------------------
# Selection: Sec. 3.1 (K highest scores) and Sec. 3.2 "Sparse Inference" (score above a threshold).
# Both return a boolean activation mask M[T,E] (the mask of Eq. 2).
# --------------------------------------------------------------------------------------------------
def select_topk(S, k: int) -> np.ndarray:
    """A(t) = the K experts with the highest scores; equal scores go to the lower index."""
    S = np.asarray(S)
    T, E = S.shape
    if not 1 <= k <= E:
        raise ValueError("k must be in [1, E]")
    # stable sort of -S keeps the lower index first among equal scores
    order = np.argsort(-S, axis=1, kind="stable")
    M = np.zeros((T, E), dtype=bool)
    np.put_along_axis(M, order[:, :k], True, axis=1)
    return M


def select_threshold(S, eps: float) -> np.ndarray:
    """A(t) = {e : S[t,e] > eps}; a token with an empty set keeps its argmax (lowest index)."""
    S = np.asarray(S)
    M = S > eps
    empty = ~M.any(axis=1)
    if empty.any():
        rows = np.nonzero(empty)[0]
        M[rows, np.argmax(S[rows], axis=1)] = True   # argmax returns the first maximum
    return M


def select(S, mode: str, k: int = 0, eps: float = 0.0) -> np.ndarray:
    if mode == "topk":
        return select_topk(S, k)
    if mode == "threshold":
        return select_threshold(S, eps)
    if mode == "threshold_topk":
        return select_threshold_topk(S, eps)
    raise ValueError(mode)


def threshold_topk_k(S, eps: float) -> int:
    """Threshold-TopK (Sec. 4.3): the batch average number of experts above the threshold, used as
    a fixed K.  Rounded half up and clamped to [1, E]."""
    M = select_threshold(S, eps)
    mean = M.sum() / M.shape[0]
    return int(min(max(np.floor(mean + 0.5), 1), M.shape[1]))


def select_threshold_topk(S, eps: float) -> np.ndarray:
    """Threshold-TopK selection (Sec. 4.3): top-K with the K that the threshold gives on this batch."""
    return select_topk(S, threshold_topk_k(S, eps))


# --------------------------------------------------------------------------------------------------
# Dispatch bookkeeping ("duplication of intermediate tokens", Sec. 4.4): the grouping of
# (token, expert) pairs by expert.  Canonical order: experts ascending, tokens ascending inside an
# expert; a token's own rows are listed in ascending expert order.
# --------------------------------------------------------------------------------------------------
@dataclass
class Routing:
    mask: np.ndarray        # [T, E] bool
    mask_bits: np.ndarray   # [T] uint64, bit e set <=> e in A(t)
    cnt_tok: np.ndarray     # [T] int32, |A(t)|
    cnt_exp: np.ndarray     # [E] int32, tokens per expert
    expert_off: np.ndarray  # [E+1] int32, exclusive prefix sum of cnt_exp
    row_token: np.ndarray   # [nnz] int32, token of each dispatched row
    row_weight: np.ndarray  # [nnz] S[token, expert] of each dispatched row
    tok_off: np.ndarray     # [T+1] int32, exclusive prefix sum of cnt_tok
    tok_rows: np.ndarray    # [nnz] int32, rows of each token in ascending expert order
    nnz: int


def dispatch(M, S) -> Routing:
    M = np.asarray(M, dtype=bool)
    S = np.asarray(S)
    T, E = M.shape
    if E > 64:
        raise ValueError("mask_bits holds at most 64 experts")
    bits = np.zeros(T, dtype=np.uint64)
    for e in range(E):
        bits |= M[:, e].astype(np.uint64) << np.uint64(e)
    cnt_tok = M.sum(axis=1).astype(np.int32)
    cnt_exp = M.sum(axis=0).astype(np.int32)
    expert_off = np.zeros(E + 1, dtype=np.int32)
    expert_off[1:] = np.cumsum(cnt_exp)
    tok_off = np.zeros(T + 1, dtype=np.int32)
    tok_off[1:] = np.cumsum(cnt_tok)
    nnz = int(expert_off[E])
    row_token = np.empty(nnz, dtype=np.int32)
    row_weight = np.empty(nnz, dtype=S.dtype)
    row_of = -np.ones((T, E), dtype=np.int64)
    for e in range(E):
        toks = np.nonzero(M[:, e])[0]                     # ascending token index
        rows = expert_off[e] + np.arange(toks.size)
        row_token[rows] = toks
        row_weight[rows] = S[toks, e]
        row_of[toks, e] = rows
    tok_rows = row_of[M].astype(np.int32)                 # row-major walk: t ascending, e ascending
    return Routing(M, bits, cnt_tok, cnt_exp, expert_off, row_token, row_weight, tok_off, tok_rows, nnz)


# --------------------------------------------------------------------------------------------------
# Expert: the MLP module e_j of Sec. 3.1, here a SwiGLU feed-forward block.
# --------------------------------------------------------------------------------------------------
def sigmoid(g):
    return 1.0 / (1.0 + np.exp(-g))


def silu(g):
    return g * sigmoid(g)


def silu_prime(g):
    s = sigmoid(g)
    return s * (1.0 + g * (1.0 - s))


def gelu(g):
    """GeLU, the activation the paper's experts use (Sec. 4.1): g * Phi(g), Phi the standard normal CDF."""
    return 0.5 * g * (1.0 + _erf(g / np.sqrt(2.0)))


def gelu_prime(g):
    """d gelu / d g = Phi(g) + g * phi(g), phi the standard normal density."""
    return 0.5 * (1.0 + _erf(g / np.sqrt(2.0))) + g * np.exp(-0.5 * g * g) / np.sqrt(2.0 * np.pi)


def _of(W, e):
    return None if W is None else W[e]


def expert_ffn(x, w_gate_e, w_up_e, w_down_e) -> np.ndarray:
    """e_j(x) for rows x[n,d].  SwiGLU expert: (silu(x W_gate) * (x W_up)) W_down.  With w_up_e = None the
    two-matrix GeLU expert of the paper (Sec. 4.1): gelu(x W_1) W_2 with W_1 = w_gate_e, W_2 = w_down_e."""
    x = _f64(x)
    g = x @ _f64(w_gate_e)
    if w_up_e is None:
        return gelu(g) @ _f64(w_down_e)
    u = x @ _f64(w_up_e)
    return (silu(g) * u) @ _f64(w_down_e)


def expert_outputs_permuted(X, r: Routing, W_gate, W_up, W_down) -> np.ndarray:
    """Y[row] = e_expert(row)(X[row_token[row]]) for every dispatched row."""
    X = _f64(X)
    E = W_gate.shape[0]
    Y = np.zeros((r.nnz, W_down.shape[2]), dtype=F64)
    for e in range(E):
        lo, hi = r.expert_off[e], r.expert_off[e + 1]
        if hi > lo:
            Y[lo:hi] = expert_ffn(X[r.row_token[lo:hi]], W_gate[e], _of(W_up, e), W_down[e])
    return Y


def combine(Y, r: Routing, T: int) -> np.ndarray:
    """O[t] = sum over the rows of t, in ascending expert order, of row_weight * Y[row] (Eq. 1)."""
    O = np.zeros((T, Y.shape[1]), dtype=F64)
    for t in range(T):
        for j in range(r.tok_off[t], r.tok_off[t + 1]):
            row = r.tok_rows[j]
            O[t] += F64(r.row_weight[row]) * Y[row]
    return O


# --------------------------------------------------------------------------------------------------
# Sparse inference forward: Eq. 1.
# --------------------------------------------------------------------------------------------------
def sparse_forward(X, W_r, b_r, W_gate, W_up, W_down, mode: str, k: int = 0, eps: float = 0.0,
                   tokens: Optional[Sequence[int]] = None):
    """O[t] = sum_{e in A(t)} S[t,e] e_e(X[t]), summed over e ascending.

    `tokens` restricts the output rows that are evaluated (each token's output depends on no other
    token); routing is always computed for every token.  Returns (O, S, mask).
    """
    X = _f64(X)
    S = route(X, W_r, b_r)
    M = select(S, mode, k, eps)
    T, E = S.shape
    tok = np.arange(T) if tokens is None else np.asarray(tokens, dtype=np.int64)
    O = np.zeros((tok.size, W_down.shape[2]), dtype=F64)
    for e in range(E):
        sel = np.nonzero(M[tok, e])[0]
        if sel.size:
            t = tok[sel]
            O[sel] += S[t, e][:, None] * expert_ffn(X[t], W_gate[e], _of(W_up, e), W_down[e])
    return O, S, M


# --------------------------------------------------------------------------------------------------
# Dense training forward (Sec. 3.2 "Dense Training"): every expert runs on every token and its
# output is retained for the backward pass.
# --------------------------------------------------------------------------------------------------
def dense_forward(X, W_r, b_r, W_gate, W_up, W_down, tokens: Optional[Sequence[int]] = None):
    """O[t] = sum_{j=1..N} S[t,j] e_j(X[t]).  Returns (O, S, Y) with Y[t,j,:] = e_j(X[t])."""
    X = _f64(X)
    S = route(X, W_r, b_r)
    T, E = S.shape
    tok = np.arange(T) if tokens is None else np.asarray(tokens, dtype=np.int64)
    Y = np.empty((tok.size, E, W_down.shape[2]), dtype=F64)
    for j in range(E):
        Y[:, j, :] = expert_ffn(X[tok], W_gate[j], _of(W_up, j), W_down[j])
    O = np.zeros((tok.size, W_down.shape[2]), dtype=F64)
    for j in range(E):
        O += S[tok, j][:, None] * Y[:, j, :]
    return O, S, Y


# --------------------------------------------------------------------------------------------------
# Dense training backward: Eq. 3 followed by the chain rule through the expert, the softmax and the
# router.
# --------------------------------------------------------------------------------------------------
def grad_scores(Y, dO) -> np.ndarray:
    """Eq. 3, first half: grad S[t,j] = < e_j(X[t]), grad O[t] >."""
    return np.einsum("tjd,td->tj", _f64(Y), _f64(dO))


def expert_backward(X, S_j, w_gate_j, w_up_j, w_down_j, dO):
    """Backward of the term S_j * e_j(X) for one expert j.

    Eq. 3, second half gives grad e_j(X) = S_j grad O; the rest is the chain rule through
    Y = H W_down, H = silu(G) * U, G = X W_gate, U = X W_up.
    Returns (dX_j, dW_gate_j, dW_up_j, dW_down_j).
    """
    X, dO = _f64(X), _f64(dO)
    wg, wu, wd = _f64(w_gate_j), _f64(w_up_j), _f64(w_down_j)
    G = X @ wg
    if wu is None:   # two-matrix GeLU expert: H = gelu(G); no W_up gradient
        dY = _f64(S_j)[:, None] * dO
        dG = (dY @ wd.T) * gelu_prime(G)
        return dG @ wg.T, X.T @ dG, None, gelu(G).T @ dY
    U = X @ wu
    H = silu(G) * U
    dY = _f64(S_j)[:, None] * dO
    dW_down = H.T @ dY
    dH = dY @ wd.T
    dU = dH * silu(G)
    dG = dH * U * silu_prime(G)
    dW_up = X.T @ dU
    dW_gate = X.T @ dG
    dX = dU @ wu.T + dG @ wg.T
    return dX, dW_gate, dW_up, dW_down


def softmax_backward(S, dS) -> np.ndarray:
    """grad Z[t,j] = S[t,j] (grad S[t,j] - sum_k S[t,k] grad S[t,k])."""
    S, dS = _f64(S), _f64(dS)
    return S * (dS - (S * dS).sum(axis=1, keepdims=True))


@dataclass
class DenseGrads:
    dX: np.ndarray
    dW_r: np.ndarray
    db_r: np.ndarray
    dW_gate: np.ndarray
    dW_up: np.ndarray
    dW_down: np.ndarray
    dS: np.ndarray
    dZ: np.ndarray


def dense_backward(X, W_r, b_r, W_gate, W_up, W_down, dO) -> DenseGrads:
    """All gradients of O = sum_j S_j e_j(X) for an upstream gradient dO."""
    X, dO = _f64(X), _f64(dO)
    _, S, Y = dense_forward(X, W_r, b_r, W_gate, W_up, W_down)
    E = S.shape[1]
    dS = grad_scores(Y, dO)
    dX = np.zeros_like(X)
    dW_gate = np.zeros(W_gate.shape, dtype=F64)
    dW_up = None if W_up is None else np.zeros(W_up.shape, dtype=F64)
    dW_down = np.zeros(W_down.shape, dtype=F64)
    for j in range(E):
        dx_j, dW_gate[j], dwu_j, dW_down[j] = expert_backward(X, S[:, j], W_gate[j], _of(W_up, j), W_down[j], dO)
        if dW_up is not None:
            dW_up[j] = dwu_j
        dX += dx_j
    dZ = softmax_backward(S, dS)
    dW_r = X.T @ dZ
    db_r = dZ.sum(axis=0)
    dX += dZ @ _f64(W_r).T
    return DenseGrads(dX, dW_r, db_r, dW_gate, dW_up, dW_down, dS, dZ)


# --------------------------------------------------------------------------------------------------
# Mutual-information loss of the router (Sec. 3.2, Eq. 4-5).
# Reading of the garbled Eq. 4: p(e_i) is the minibatch mean of S_i, and H(e|X) is the entropy of
# one token's score vector.
# --------------------------------------------------------------------------------------------------
def mi_loss(S) -> float:
    S = _f64(S)
    p = S.mean(axis=0)
    with np.errstate(divide="ignore", invalid="ignore"):
        h_e = -np.sum(np.where(p > 0, p * np.log(p), 0.0))
        h_e_x = -np.sum(np.where(S > 0, S * np.log(S), 0.0), axis=1)
    return float(-h_e + h_e_x.mean())


def mi_loss_grad(S) -> np.ndarray:
    """d L_MI / d S[t,i] = (log p_i - log S[t,i]) / T  (the +1 and -1 terms cancel)."""
    S = _f64(S)
    p = S.mean(axis=0)
    return (np.log(p)[None, :] - np.log(S)) / S.shape[0]


def mi_backward(X, W_r, b_r, alpha: float):
    """Gradients of alpha * L_MI(softmax(X W_r + b_r)) w.r.t. X, W_r and b_r: the term the total loss
    L = L_LM + alpha L_MI (Sec. 3.2, Eq. 6) adds to the router's gradients.  Chain rule only: the
    gradient w.r.t. the scores goes through the softmax (Eq. 1) and the linear router."""
    X = _f64(X)
    S = route(X, W_r, b_r)
    dZ = softmax_backward(S, alpha * mi_loss_grad(S))
    return dZ @ _f64(W_r).T, X.T @ dZ, dZ.sum(axis=0)
