"""Parameter-free hyper-encoder (oracle; test infrastructure).

Section 2.2 of the paper maps the embeddings of a hypertoken's constituent base
tokens, padded to M slots, to one d-vector.  The variant computed here is the
"Averaging" row of the hyper-encoder ablation table: the mean of the constituent
base embeddings.  Padding slots contribute nothing and are not counted in the
divisor (the mean is over the entry's actual length L).  The second pooling
kind is a benchmark variant, not the paper's: a position-weighted sum with
weights softmax-normalised over the first L raw weights.

Arithmetic is float64 from the stored (float32 or bf16) table, followed by one
round-to-nearest-even into the storage format; that rounded row is what the
logit stage consumes.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np

from .numfmt import round_to_storage, to_f64


def pool_coefficients(L: int, pool: str, w: Sequence[float]) -> np.ndarray:
    """float64 [L] coefficients a_j with sum 1: 1/L (mean) or softmax(w[:L]) (weighted)."""
    if pool == "mean":
        return np.full(L, 1.0 / L, dtype=np.float64)
    if pool == "weighted":
        ww = np.asarray(w[:L], dtype=np.float64)
        e = np.exp(ww - ww.max())
        return e / e.sum()
    raise ValueError(pool)


def hyper_embed(E: np.ndarray, dtype: str, entries: Sequence[Tuple[int, ...]], cap: int,
                pool: str = "mean", w: Sequence[float] = ()) -> np.ndarray:
    """W_hyper [cap, d] in the storage format; rows at and beyond len(entries) are zero."""
    d = E.shape[1]
    out64 = np.zeros((cap, d), dtype=np.float64)
    for i, e in enumerate(entries):
        a = pool_coefficients(len(e), pool, w)
        acc = np.zeros(d, dtype=np.float64)
        for j, t in enumerate(e):
            acc += a[j] * to_f64(E[t], dtype)
        out64[i] = acc
    return round_to_storage(out64, dtype)
