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


# ---------------------------------------------------------------------------------------------------------
# Gradient of the learned hyper-encoder (training f_phi together with the model, section 2.4: the loss over
# the compressed sequence reaches phi through every hypertoken vector it produced).  Plain reverse-mode
# differentiation of encode_entry, step by step in the reverse order of the forward pass.
# ---------------------------------------------------------------------------------------------------------

def layer_norm_backward(dN: np.ndarray, x: np.ndarray, gamma: np.ndarray, eps: float = EPS):
    """N = (x - mu) / sqrt(var + eps) * gamma + beta  ->  (dx, dgamma, dbeta)."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xh = (x - mu) * rstd
    g = dN * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True) - xh * (g * xh).mean(axis=-1, keepdims=True))
    return dx, (dN * xh).sum(axis=0), dN.sum(axis=0)


def gelu_grad(x: np.ndarray) -> np.ndarray:
    """d/dx of 0.5 x (1 + erf(x / sqrt 2)) = Phi(x) + x phi(x)."""
    return 0.5 * (1.0 + erf(x / np.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)


def attention_backward(dOut: np.ndarray, A: np.ndarray, w_qkv: np.ndarray, b_qkv: np.ndarray, w_o: np.ndarray,
                       n_heads: int):
    """Backward of attention(): dOut [L, d] -> (dA, dw_qkv, db_qkv, dw_o, db_o)."""
    L, d = A.shape
    dh = d // n_heads
    qkv = A @ w_qkv.T + b_qkv
    Q, K, V = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    O = np.empty((L, d), dtype=np.float64)
    P_all = []
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        S = Q[:, sl] @ K[:, sl].T / np.sqrt(dh)
        S = S - S.max(axis=1, keepdims=True)
        Pm = np.exp(S)
        Pm /= Pm.sum(axis=1, keepdims=True)
        P_all.append(Pm)
        O[:, sl] = Pm @ V[:, sl]
    dw_o = dOut.T @ O
    db_o = dOut.sum(axis=0)
    dO = dOut @ w_o
    dqkv = np.zeros_like(qkv)
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        Pm = P_all[h]
        dP = dO[:, sl] @ V[:, sl].T
        dV = Pm.T @ dO[:, sl]
        dS = Pm * (dP - (dP * Pm).sum(axis=1, keepdims=True))
        dqkv[:, sl] = dS @ K[:, sl] / np.sqrt(dh)
        dqkv[:, d + h * dh:d + (h + 1) * dh] = dS.T @ Q[:, sl] / np.sqrt(dh)
        dqkv[:, 2 * d + h * dh:2 * d + (h + 1) * dh] = dV
    return dqkv @ w_qkv, dqkv.T @ A, dqkv.sum(axis=0), dw_o, db_o


def zero_grads(enc64: dict) -> dict:
    return dict(pos=None if enc64["pos"] is None else np.zeros_like(enc64["pos"]),
                layers=[{k: np.zeros_like(v) for k, v in lay.items()} for lay in enc64["layers"]])


def encode_entry_backward(X0: np.ndarray, enc64: dict, dh_out: np.ndarray, grads: dict) -> np.ndarray:
    """Adds the entry's parameter gradients to `grads` (as made by zero_grads) and returns dX0 [L, d], given
    dh_out = dLoss / d encode_entry(X0)."""
    xs = []                      # forward, keeping each layer's input and middle state
    X = X0
    for lay in enc64["layers"]:
        A = layer_norm(X, lay["ln1_g"], lay["ln1_b"])
        Y = X + attention(A, lay["w_qkv"], lay["b_qkv"], lay["w_o"], lay["b_o"], enc64["n_heads"])
        xs.append((X, A, Y))
        X = Y
        if not enc64["attention_only"]:
            N2 = layer_norm(Y, lay["ln2_g"], lay["ln2_b"])
            U = N2 @ lay["w_1"].T + lay["b_1"]
            X = Y + gelu(U) @ lay["w_2"].T + lay["b_2"]
    L = X0.shape[0]
    dX = np.tile(dh_out / L, (L, 1))             # h = mean over the L real slots
    for lay, g, (Xin, A, Y) in zip(reversed(enc64["layers"]), reversed(grads["layers"]), reversed(xs)):
        dY = dX
        if not enc64["attention_only"]:
            N2 = layer_norm(Y, lay["ln2_g"], lay["ln2_b"])
            U = N2 @ lay["w_1"].T + lay["b_1"]
            F = gelu(U)
            g["w_2"] += dX.T @ F
            g["b_2"] += dX.sum(axis=0)
            dU = (dX @ lay["w_2"]) * gelu_grad(U)
            g["w_1"] += dU.T @ N2
            g["b_1"] += dU.sum(axis=0)
            dYn, dg, db = layer_norm_backward(dU @ lay["w_1"], Y, lay["ln2_g"])
            g["ln2_g"] += dg
            g["ln2_b"] += db
            dY = dX + dYn
        dA, dwqkv, dbqkv, dwo, dbo = attention_backward(dY, A, lay["w_qkv"], lay["b_qkv"], lay["w_o"],
                                                        enc64["n_heads"])
        g["w_qkv"] += dwqkv
        g["b_qkv"] += dbqkv
        g["w_o"] += dwo
        g["b_o"] += dbo
        dXn, dg, db = layer_norm_backward(dA, Xin, lay["ln1_g"])
        g["ln1_g"] += dg
        g["ln1_b"] += db
        dX = dY + dXn
    return dX


def hyper_encode_backward(E: np.ndarray, dtype: str, entries: Sequence[Tuple[int, ...]], enc: dict,
                          dW_hyper: np.ndarray) -> dict:
    """Gradient of  sum_{i, k} dW_hyper[i, k] * f_phi(entries[i])[k]  for ONE sequence's entries (float64, taken
    at the unrounded forward values): dict(dE [V, d], pos [M, d] or None, layers: list of dicts keyed like the
    encoder's layers).  A token that occurs in several slots receives every slot's gradient."""
    e64 = widen_encoder(enc, dtype)
    grads = zero_grads(e64)
    dE = np.zeros((E.shape[0], E.shape[1]), dtype=np.float64)
    for i, e in enumerate(entries):
        X = np.stack([to_f64(E[t], dtype) for t in e])
        if e64["pos"] is not None:
            X = X + e64["pos"][:len(e)]
        dX0 = encode_entry_backward(X, e64, np.asarray(dW_hyper[i], dtype=np.float64), grads)
        for j, t in enumerate(e):
            dE[t] += dX0[j]
        if grads["pos"] is not None:
            grads["pos"][:len(e)] += dX0
    return dict(dE=dE, pos=grads["pos"], layers=grads["layers"])
