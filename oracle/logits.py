"""Joint logits over the base and hyper vocabularies (oracle; test infrastructure).

Section 2.3, steps 7-9: the hypertoken unembedding rows are appended to the
language-model head, one softmax is taken over the union, and the next token is
chosen from it.  For the rows of one sequence:

    logits[r, v] = sum_k H[r, k] * W[v, k],   W = [W_base ; W_hyper[:C]]

Only the C existing hypertokens are columns; unused slots do not exist (they
can never be predicted).  Per row the oracle returns the maximum, its index
(lowest index on exact ties), the log-sum-exp (natural log) and the gap between
the two largest logits.  Everything is float64 on the exactly widened inputs.
"""
from __future__ import annotations

import numpy as np

from .numfmt import to_f64


def extended_logits(H: np.ndarray, W_base: np.ndarray, W_hyper: np.ndarray, C: int, dtype: str,
                    return_logits: bool = True, block: int = 8192) -> dict:
    """H [rows, d] (rows of ONE sequence), W_base [V, d], W_hyper [cap, d] of that sequence, C entries."""
    Hd = to_f64(H, dtype)
    rows = Hd.shape[0]
    V = W_base.shape[0]
    n_cols = V + int(C)
    logits = np.empty((rows, n_cols), dtype=np.float64)
    for v0 in range(0, V, block):
        v1 = min(V, v0 + block)
        logits[:, v0:v1] = Hd @ to_f64(W_base[v0:v1], dtype).T
    for c0 in range(0, int(C), block):
        c1 = min(int(C), c0 + block)
        logits[:, V + c0:V + c1] = Hd @ to_f64(W_hyper[c0:c1], dtype).T
    mx = logits.max(axis=1)
    am = logits.argmax(axis=1)
    lse = mx + np.log(np.exp(logits - mx[:, None]).sum(axis=1))
    if n_cols > 1:
        top2 = np.partition(logits, n_cols - 2, axis=1)[:, n_cols - 2]
        margin = mx - top2
    else:
        margin = np.full(rows, np.inf)
    out = dict(argmax=am.astype(np.int64), max=mx, lse=lse, margin=margin)
    if return_logits:
        out["logits"] = logits
    return out
