"""Test-side helpers: margin conditioning of synthetic inputs and error metrics.

Margin conditioning: the GPU computes router scores in fp32 with its own summation order, the
checker in fp64.  A token whose selection would flip under a relative perturbation of `tau` of a
score (a score within tau*eps of the threshold, or a K-th / (K+1)-th score gap below tau*score) is
redrawn, so that the selected sets are well defined for any faithful implementation.  The scores
used for this come from the CPU checker, never from the GPU.
"""
import numpy as np

import dsmoe_inputs as gen
from oracle import dsmoe_oracle as orc

TAU = 1e-3


def unsafe_tokens(S, mode, k, eps, tau=TAU):
    if mode == "threshold_topk":
        # both decisions must be safe: the counts that give K, and the top-K at that K
        a = unsafe_tokens(S, "threshold", 0, eps, tau)
        b = unsafe_tokens(S, "topk", orc.threshold_topk_k(S, eps), 0.0, tau)
        return np.union1d(a, b)
    if mode == "threshold":
        return np.nonzero((np.abs(S - eps) < tau * eps).any(axis=1))[0]
    E = S.shape[1]
    if k >= E:
        return np.zeros(0, dtype=np.int64)
    srt = -np.sort(-S, axis=1)
    return np.nonzero((srt[:, k - 1] - srt[:, k]) < tau * srt[:, k - 1])[0]


def condition_margins(inp, mode, k=0, eps=0.0, tau=TAU, max_rounds=64):
    """Redraw tokens of `inp.x` in place until no selection decision sits inside the margin."""
    S = orc.route(inp.x, inp.w_r, inp.b_r)
    total = 0
    for _ in range(max_rounds):
        bad = unsafe_tokens(S, mode, k, eps, tau)
        if bad.size == 0:
            return total
        total += bad.size
        gen.redraw_rows(inp, bad)
        S[bad] = orc.route(inp.x[bad], inp.w_r, inp.b_r)
    raise RuntimeError("margin conditioning did not converge")


def rel_err(got, ref):
    """max|got - ref| / max|ref| (the layer's parity metric)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))
