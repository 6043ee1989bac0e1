"""CPU checker for the Mixture-of-Attention-heads (MoA) layer of DS-MoE: the plain definition in fp64.

TEST INFRASTRUCTURE ONLY.  Imported by the test-suite (and nothing in the product); shares no code with
the HIP path.  The router and the expert selection are those of the MLP layer and are taken from the
sibling checker module.

Definition (Sec. 3.2, "Mixture of Attention Head", Eq. 7-8).  N experts; expert i owns a query projection
W_q[i] (d_h -> N_head * d_head) and an output projection W_o[i] (N_head * d_head -> d_h); the N_head
key/value heads K[j], V[j] (a cache of L positions) are shared by all experts (grouped-query attention:
head j of every expert attends to K[j], V[j]).  For a token X with router scores S and selected set A:

    Q_i   = X W_q[i]                                            (N_head vectors of d_head)
    O_ij  = softmax(scale * Q_ij K_j^T) V_j W_o[i][j]            (Eq. 7)
    O     = sum_{i in A} S_i sum_j O_ij                          (Eq. 8)

Array shapes: X[T,d], W_r[d,E], W_q[E,d,N_head*d_head], K[N_head,L,d_head], V[N_head,L,d_head],
W_o[E,N_head*d_head,d].

Readings taken where the paper is silent (listed in the design notes):
  * Eq. 7 prints softmax(Q K^T) without a factor; `scale` is an argument (1 reproduces the print,
    1/sqrt(d_head) is the usual attention);
  * language-model attention is causal: the T tokens are the last T positions of the cache
    (position of token t = L - T + t) and a token attends to cache positions <= its own;
  * the kept scores weigh the expert outputs as they are (no renormalisation), as in Eq. 1.

Pinned by tests that do not call these functions for their expected values: scalar brute force,
scipy's softmax on a one-expert one-head case, closed forms (constant values, zero scale), causality
and invariance checks.
"""
from __future__ import annotations

import numpy as np

from . import dsmoe_oracle as moe

F64 = np.float64


def _f64(a):
    return None if a is None else np.asarray(a, dtype=F64)


def attention_head(Q, K_j, V_j, pos0: int, scale: float) -> np.ndarray:
    """softmax(scale * Q K_j^T) V_j of Eq. 7 for one head: Q[T,d_head], K_j, V_j[L,d_head]; query t sees cache
    positions 0 .. pos0 + t."""
    Q, K_j, V_j = _f64(Q), _f64(K_j), _f64(V_j)
    T, L = Q.shape[0], K_j.shape[0]
    A = scale * (Q @ K_j.T)                                          # [T, L]
    visible = np.arange(L)[None, :] <= (pos0 + np.arange(T))[:, None]
    A = np.where(visible, A, -np.inf)
    A = A - A.max(axis=1, keepdims=True)
    P = np.exp(A)
    P = P / P.sum(axis=1, keepdims=True)
    return P @ V_j


def expert_heads(X, W_q_i, K, V, W_o_i, pos0: int, scale: float) -> np.ndarray:
    """sum_j O_ij of Eq. 7-8 for one expert i and every token: [T, d]."""
    X, W_q_i, W_o_i = _f64(X), _f64(W_q_i), _f64(W_o_i)
    n_head, d_head = K.shape[0], K.shape[2]
    Qi = X @ W_q_i                                                   # [T, N_head * d_head]
    out = np.zeros((X.shape[0], W_o_i.shape[1]), dtype=F64)
    for j in range(n_head):
        cols = slice(j * d_head, (j + 1) * d_head)
        C = attention_head(Qi[:, cols], K[j], V[j], pos0, scale)    # [T, d_head]
        out += C @ W_o_i[cols, :]
    return out


def moa_forward(X, W_r, b_r, W_q, K, V, W_o, mode: str, k: int = 0, eps: float = 0.0, scale: float = 1.0):
    """Eq. 8.  mode: "dense" (A = all experts), "topk", "threshold", "threshold_topk" as in the MLP layer.
    Returns (O[T,d], S[T,E], M[T,E] bool)."""
    X = _f64(X)
    T, E, L = X.shape[0], W_q.shape[0], K.shape[1]
    pos0 = L - T
    if pos0 < 0:
        raise ValueError("the cache holds the T tokens themselves: L >= T")
    S = moe.route(X, W_r, b_r)
    M = np.ones((T, E), dtype=bool) if mode == "dense" else moe.select(S, mode, k, eps)
    O = np.zeros((T, W_o.shape[2]), dtype=F64)
    for i in range(E):
        Oi = expert_heads(X, W_q[i], K, V, W_o[i], pos0, scale)
        O += (S[:, i] * M[:, i])[:, None] * Oi
    return O, S, M


# --------------------------------------------------------------------------------------------------
# Dense training of the attention layer: every expert active, weighted by its score (Sec. 3.2, "Dense
# Training"), and the gradients of that forward.  The score gradient follows Eq. 3 with the attention
# experts in the place of the MLP experts; the rest is the chain rule through Eq. 7.
# --------------------------------------------------------------------------------------------------
def _attention_probs(Q, K_j, pos0: int, scale: float) -> np.ndarray:
    T, L = Q.shape[0], K_j.shape[0]
    A = scale * (Q @ K_j.T)
    visible = np.arange(L)[None, :] <= (pos0 + np.arange(T))[:, None]
    A = np.where(visible, A, -np.inf)
    A = A - A.max(axis=1, keepdims=True)
    P = np.exp(A)
    return P / P.sum(axis=1, keepdims=True)


def moa_dense_backward(X, W_r, b_r, W_q, K, V, W_o, dO, scale: float = 1.0):
    """Gradients of O = sum_i S_i sum_j O_ij (all experts) with respect to X, W_r, b_r, W_q, W_o and the cache
    K, V, for the upstream gradient dO[T,d].  Returns a dict of arrays shaped like their tensors."""
    X, W_r, W_q, K, V, W_o, dO = (_f64(a) for a in (X, W_r, W_q, K, V, W_o, dO))
    T, d = X.shape
    E, n_head, L, d_head = W_q.shape[0], K.shape[0], K.shape[1], K.shape[2]
    pos0 = L - T
    S = moe.route(X, W_r, b_r)
    dX = np.zeros_like(X)
    dW_q, dW_o = np.zeros_like(W_q), np.zeros_like(W_o)
    dK, dV = np.zeros_like(K), np.zeros_like(V)
    dS = np.zeros_like(S)
    for i in range(E):
        Qi = X @ W_q[i]
        dQi = np.zeros_like(Qi)
        out_i = np.zeros((T, d), dtype=F64)                    # e_i(X) = sum_j O_ij
        dE = S[:, i][:, None] * dO                             # gradient reaching the expert's output
        for j in range(n_head):
            cols = slice(j * d_head, (j + 1) * d_head)
            P = _attention_probs(Qi[:, cols], K[j], pos0, scale)
            C = P @ V[j]
            out_i += C @ W_o[i][cols, :]
            dW_o[i][cols, :] += C.T @ dE
            dC = dE @ W_o[i][cols, :].T
            dV[j] += P.T @ dC
            dP = dC @ V[j].T
            dA = P * (dP - (dP * P).sum(axis=1, keepdims=True))   # softmax backward, row by row
            dQi[:, cols] = scale * (dA @ K[j])
            dK[j] += scale * (dA.T @ Qi[:, cols])
        dS[:, i] = (out_i * dO).sum(axis=1)                    # Eq. 3: grad S_i = <e_i(X), dO>
        dW_q[i] = X.T @ dQi
        dX += dQi @ W_q[i].T
    dZ = S * (dS - (dS * S).sum(axis=1, keepdims=True))
    dX += dZ @ W_r.T
    return dict(dX=dX, dW_r=X.T @ dZ, db_r=dZ.sum(axis=0), dW_q=dW_q, dW_o=dW_o, dK=dK, dV=dV, dS=dS)
