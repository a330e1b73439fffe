"""Learned hyper-encoder (oracle; test infrastructure).

Section 2.2 of the zip2zip paper: a hypertoken's vector is produced by a small
network f_phi from the embeddings of its constituent base tokens, padded to M
slots.  The hyper-encoder ablation (appendix "Discussions on Hyper-Encoder
Architecture", table of architectures) names the variants "averaging",
"1-attention-layer", "1-transformer-layer" and "2-transformer-layer"; the
training setup (section 4.2) uses the two-layer transformer encoder with
M = 3.  The paper gives no further detail of these networks.  The reading
taken here, layer by layer, is the standard pre-norm transformer encoder:

    X_i   = E[y_i] + P_i                      i < L  (P: learned slot positions, optional)
    A     = LayerNorm_1(X)
    Q,K,V = A Wq^T + bq,  A Wk^T + bk,  A Wv^T + bv          (Wq, Wk, Wv stacked as w_qkv [3d, d])
    per head h (width d / n_heads):
        S = Q_h K_h^T / sqrt(d / n_heads)      over the L real slots only (padding is masked out as keys)
        O_h = softmax_rows(S) V_h
    Y     = X + O Wo^T + bo                                   -- "attention layer"
    Z     = Y + GELU(LayerNorm_2(Y) W1^T + b1) W2^T + b2      -- "transformer layer" (GELU with erf)
    h     = mean over the L real slots of the last layer's output

LayerNorm is over the d features with the biased variance and eps inside the
square root.  Padding slots are never keys and never enter the mean, so the
network is evaluated on the L real slots alone; M only bounds L and sizes P.

Matrices are stored in the model's storage format (float32 or bf16 bit
patterns, [out, in] row-major), vectors (biases, LayerNorm scale and shift) in
float32.  Arithmetic is float64 throughout with one round-to-nearest-even of
h into the storage format at the end.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np
from scipy.special import erf

from .numfmt import round_to_storage, to_f64

EPS = 1e-5


def layer_norm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float = EPS) -> np.ndarray:
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma + beta


def gelu(x: np.ndarray) -> np.ndarray:
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def attention(A: np.ndarray, w_qkv: np.ndarray, b_qkv: np.ndarray, w_o: np.ndarray, b_o: np.ndarray,
              n_heads: int) -> np.ndarray:
    """Multi-head self-attention among the rows of A [L, d] (all of them real slots), output projection included."""
    L, d = A.shape
    dh = d // n_heads
    qkv = A @ w_qkv.T + b_qkv                       # [L, 3d]
    Q, K, V = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    O = np.empty((L, d), dtype=np.float64)
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        S = Q[:, sl] @ K[:, sl].T / np.sqrt(dh)     # [L, L]
        S = S - S.max(axis=1, keepdims=True)
        Pm = np.exp(S)
        Pm /= Pm.sum(axis=1, keepdims=True)
        O[:, sl] = Pm @ V[:, sl]
    return O @ w_o.T + b_o


def widen_encoder(enc: dict, dtype: str) -> dict:
    """The encoder's parameters as float64 arrays (exact widening of what is stored)."""
    out = dict(n_heads=int(enc["n_heads"]), attention_only=bool(enc["attention_only"]),
               pos=None if enc.get("pos") is None else to_f64(enc["pos"], dtype), layers=[])
    for lay in enc["layers"]:
        w = {}
        for k, v in lay.items():
            w[k] = to_f64(v, dtype) if k.startswith("w_") else np.asarray(v, dtype=np.float32).astype(np.float64)
        out["layers"].append(w)
    return out


def encode_entry(X: np.ndarray, enc64: dict) -> np.ndarray:
    """f_phi on one entry: X [L, d] float64 (embeddings plus positions of the real slots) -> h [d]."""
    for lay in enc64["layers"]:
        A = layer_norm(X, lay["ln1_g"], lay["ln1_b"])
        X = X + attention(A, lay["w_qkv"], lay["b_qkv"], lay["w_o"], lay["b_o"], enc64["n_heads"])
        if not enc64["attention_only"]:
            F = gelu(layer_norm(X, lay["ln2_g"], lay["ln2_b"]) @ lay["w_1"].T + lay["b_1"])
            X = X + F @ lay["w_2"].T + lay["b_2"]
    return X.mean(axis=0)


def hyper_encode(E: np.ndarray, dtype: str, entries: Sequence[Tuple[int, ...]], cap: int, enc: dict,
                 rounded: bool = True) -> np.ndarray:
    """W_hyper [cap, d]: row i = f_phi(entries[i]); rows at and beyond len(entries) are zero.  In the storage
    format, or float64 before the final rounding with rounded=False."""
    d = E.shape[1]
    e64 = widen_encoder(enc, dtype)
    out64 = np.zeros((cap, d), dtype=np.float64)
    for i, e in enumerate(entries):
        X = np.stack([to_f64(E[t], dtype) for t in e])
        if e64["pos"] is not None:
            X = X + e64["pos"][:len(e)]
        out64[i] = encode_entry(X, e64)
    return round_to_storage(out64, dtype) if rounded else out64
