"""Negative log-likelihood of target codes under the joint softmax (oracle; test infrastructure).

Section 2.4 of the zip2zip paper trains with the usual next-token objective, taken over the compressed
sequence (its second displayed equation): every position contributes -log of the probability the joint
softmax over base tokens and hypertokens gives to the code that actually follows.  For hidden row r with
target code t (a base token, or V + e for entry e of the row's sequence):

    nll[r] = log-sum-exp_v(logits[r, v]) - logits[r, t]

over the V + C existing columns.  A negative target marks a position without a target (it contributes 0);
a target that names no existing column has probability zero (nll = +inf).
"""
from __future__ import annotations

import numpy as np

from .logits import extended_logits


def extended_nll(H: np.ndarray, W_base: np.ndarray, W_hyper: np.ndarray, C: int, dtype: str,
                 targets: np.ndarray) -> dict:
    """Rows of ONE sequence.  Returns dict(nll float64 [rows], lse float64 [rows])."""
    r = extended_logits(H, W_base, W_hyper, C, dtype, return_logits=True)
    lg, lse = r["logits"], r["lse"]
    n_cols = lg.shape[1]
    nll = np.zeros(lg.shape[0], dtype=np.float64)
    for i, t in enumerate(np.asarray(targets).tolist()):
        if t < 0:
            nll[i] = 0.0
        elif t >= n_cols:
            nll[i] = np.inf
        else:
            nll[i] = lse[i] - lg[i, t]
    return dict(nll=nll, lse=lse)


def extended_nll_backward(H: np.ndarray, W_base: np.ndarray, W_hyper: np.ndarray, C: int, dtype: str,
                          targets: np.ndarray, grad_nll: np.ndarray) -> dict:
    """Gradient of sum_r grad_nll[r] * nll[r] for the rows of ONE sequence (float64).

    With p = softmax(logits[r, :]) over the V + C existing columns and t the row's target,
    d nll[r] / d logits[r, v] = p[v] - [v == t].  Rows without a target (t < 0) and rows whose target names
    no existing column (nll = +inf: no finite gradient) contribute nothing.  From dZ = grad_nll[:, None] *
    (P - onehot):  dH = dZ W,  dW_base = dZ[:, :V]^T H,  dW_hyper[:C] = dZ[:, V:]^T H  (rows at and beyond C: 0).
    """
    from .numfmt import to_f64

    r = extended_logits(H, W_base, W_hyper, C, dtype, return_logits=True)
    lg, lse = r["logits"], r["lse"]
    V = W_base.shape[0]
    n_cols = lg.shape[1]
    H64, Wb, Wh = to_f64(H, dtype), to_f64(W_base, dtype), to_f64(W_hyper, dtype)
    dZ = np.exp(lg - lse[:, None])
    g = np.asarray(grad_nll, dtype=np.float64).copy()
    for i, t in enumerate(np.asarray(targets).tolist()):
        if 0 <= t < n_cols:
            dZ[i, t] -= 1.0
        else:
            g[i] = 0.0
    dZ *= g[:, None]
    W = np.concatenate([Wb, Wh[:C]])
    dWh = np.zeros_like(Wh)
    dWh[:C] = dZ[:, V:].T @ H64
    return dict(dH=dZ @ W, dW_base=dZ[:, :V].T @ H64, dW_hyper=dWh, dZ=dZ)


def hyper_embed_backward(dW_hyper: np.ndarray, entries, V: int, pool: str = "mean", w=()) -> np.ndarray:
    """Gradient through the pooling of ONE sequence's entries (float64): W_hyper[e] = sum_j a_j E[t_j], so
    dE[t_j] += a_j * dW_hyper[e] for every token of every entry (a token that occurs twice receives twice)."""
    from .embed import pool_coefficients

    dE = np.zeros((V, dW_hyper.shape[1]), dtype=np.float64)
    for e, toks in enumerate(entries):
        a = pool_coefficients(len(toks), pool, w)
        for j, t in enumerate(toks):
            dE[t] += a[j] * dW_hyper[e]
    return dE
