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
