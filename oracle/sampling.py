"""Sampling the next token from the joint softmax (oracle; test infrastructure).

Section 2.3, steps 8-9 of the zip2zip paper: the model's next token is a draw
from the joint softmax over base tokens and hypertokens.  The paper names no
sampler; the reading taken here is temperature sampling,

    token ~ softmax(logits / T)        over the V + C existing columns,

realised with the Gumbel-max construction: with g_v = -ln(-ln u_v) and u_v
independent uniforms on (0, 1), argmax_v (logits_v / T + g_v) is distributed
exactly as softmax(logits / T).  The uniforms are a pure function of
(seed, step, hidden row, column) through the counter-based generator
Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
1, 2, 3", SC'11), so that this oracle and the HIP path draw the same numbers
while sharing no code.  Layout of one draw:

    counter = (column >> 2, hidden row, step & 0xffffffff, step >> 32)
    key     = (seed & 0xffffffff, seed >> 32)
    word    = output[column & 3]
    u       = ((word >> 9) + 0.5) * 2**-23          (an odd multiple of 2**-24: exact in float32)

Truncation (the usual top-k / nucleus filters, a reading as well): order the columns by logit / T,
largest first, equal values by lower column.  With q = softmax(logits / T) over all existing columns,
keep the first n columns of that order, n = min(k, n_p), where n_p is the smallest prefix whose q sums
to at least p (both filters look at the full distribution; k <= 0 and p >= 1 switch a filter off; at least
one column is kept).  The draw is the Gumbel-max over the kept columns with the same uniforms, i.e. a
draw from q renormalised on the kept set.

Besides the drawn column the oracle returns its log-probability under
softmax(logits / T) and the gap between the two largest perturbed values (a
draw is only comparable between two implementations when that gap exceeds
their rounding differences).
"""
from __future__ import annotations

import numpy as np

from .logits import extended_logits

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH = np.uint64(32)


def philox4x32_10(counter, key):
    """Ten rounds of Philox-4x32.  counter: array-like [..., 4] of 32-bit words, key: two 32-bit words
    (scalars or arrays broadcastable to counter[..., 0]).  Returns uint32 [..., 4]."""
    c = np.asarray(counter, dtype=np.uint64) & _MASK
    c0, c1, c2, c3 = (c[..., i].copy() for i in range(4))
    k0 = np.asarray(key[0], dtype=np.uint64) & _MASK
    k1 = np.asarray(key[1], dtype=np.uint64) & _MASK
    for r in range(10):
        if r > 0:                                   # the key schedule: a Weyl sequence per round
            k0 = (k0 + np.uint64(_W0)) & _MASK
            k1 = (k1 + np.uint64(_W1)) & _MASK
        p0 = _M0 * c0                               # 32 x 32 -> 64 bit products
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH, p0 & _MASK
        hi1, lo1 = p1 >> _SH, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def uniforms(seed: int, step: int, row: int, n_cols: int) -> np.ndarray:
    """u[v] for columns 0..n_cols-1 of one hidden row, float64, each an odd multiple of 2**-24 in (0, 1)."""
    groups = (n_cols + 3) // 4
    ctr = np.empty((groups, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(groups, dtype=np.uint64)
    ctr[:, 1] = np.uint64(row & 0xFFFFFFFF)
    ctr[:, 2] = np.uint64(step & 0xFFFFFFFF)
    ctr[:, 3] = np.uint64((step >> 32) & 0xFFFFFFFF)
    words = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)).reshape(-1)[:n_cols]
    return ((words >> np.uint32(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def gumbel(u: np.ndarray) -> np.ndarray:
    return -np.log(-np.log(u))


def sample_row(logits: np.ndarray, temperature: float, seed: int, step: int, row: int) -> dict:
    """One draw from softmax(logits / temperature) for one hidden row (logits: float64 [n_cols])."""
    z = logits / float(temperature)
    pert = z + gumbel(uniforms(seed, step, row, z.shape[0]))
    tok = int(np.argmax(pert))                      # lowest column on exact ties
    m = z.max()
    lse = m + np.log(np.exp(z - m).sum())
    if z.shape[0] > 1:
        part = np.partition(pert, z.shape[0] - 2)
        gap = float(part[-1] - part[-2])
    else:
        gap = float("inf")
    return dict(token=tok, logprob=float(z[tok] - lse), gap=gap, lse=float(lse), perturbed=pert)


def kept_prefix(z: np.ndarray, top_k: int, top_p: float) -> dict:
    """The truncation rule on one row of scaled logits z (float64).  Returns the kept columns (in order),
    and how close the rule came to deciding otherwise: `order_gap` = z of the last kept column minus z of
    the first dropped one (inf if nothing is dropped), `mass_gap` = distance of the cumulative probability
    from top_p at the decisive prefixes (inf when the nucleus filter is off)."""
    n_cols = z.shape[0]
    order = np.lexsort((np.arange(n_cols), -z))          # by -z, then by column
    m = z.max()
    w = np.exp(z[order] - m)
    cum = np.cumsum(w) / w.sum()
    n_k = n_cols if top_k <= 0 else min(int(top_k), n_cols)
    if top_p >= 1.0:
        n_p, mass_gap = n_cols, float("inf")
    else:
        n_p = int(np.searchsorted(cum, top_p, side="left")) + 1      # smallest n with cum[n-1] >= p
        n_p = min(n_p, n_cols)
        below = cum[n_p - 2] if n_p >= 2 else 0.0
        mass_gap = float(min(cum[n_p - 1] - top_p, top_p - below))
    n = max(1, min(n_k, n_p))
    order_gap = float(z[order[n - 1]] - z[order[n]]) if n < n_cols else float("inf")
    if n_k < n_p:
        mass_gap = float("inf")                                      # the nucleus filter did not decide
    return dict(kept=order[:n], n=n, order_gap=order_gap, mass_gap=mass_gap)


def sample_row_truncated(logits: np.ndarray, temperature: float, top_k: int, top_p: float, seed: int, step: int,
                         row: int) -> dict:
    """One draw from softmax(logits / temperature) truncated by top_k / top_p (see the module text)."""
    z = logits / float(temperature)
    kp = kept_prefix(z, top_k, top_p)
    kept = kp["kept"]
    pert = z + gumbel(uniforms(seed, step, row, z.shape[0]))
    pk = pert[kept]
    best = pk.max()
    tok = int(kept[pk == best].min())                   # lowest column on exact ties
    m = z[kept].max()
    lse = m + np.log(np.exp(z[kept] - m).sum())
    srt = np.sort(pk)
    gap = float(srt[-1] - srt[-2]) if len(pk) > 1 else float("inf")
    return dict(token=tok, logprob=float(z[tok] - lse), gap=gap, n_kept=kp["n"], kept=kept,
                order_gap=kp["order_gap"], mass_gap=kp["mass_gap"], perturbed=pert)


def extended_sample(H: np.ndarray, W_base: np.ndarray, W_hyper: np.ndarray, C: int, dtype: str,
                    temperature: float, seed: int, step: int, row0: int) -> dict:
    """Draws for the hidden rows of ONE sequence (global row numbers row0, row0 + 1, ...) from the joint
    softmax of `extended_logits` at the given temperature.  Returns arrays token, logprob, gap."""
    lg = extended_logits(H, W_base, W_hyper, C, dtype, return_logits=True)["logits"]
    out = [sample_row(lg[i], temperature, seed, step, row0 + i) for i in range(lg.shape[0])]
    return dict(token=np.array([o["token"] for o in out], dtype=np.int64),
                logprob=np.array([o["logprob"] for o in out]),
                gap=np.array([o["gap"] for o in out]),
                logits=lg)
