"""Seeded synthetic inputs for the zip2zip dynamic-vocabulary path.

This module only draws random numbers and shapes them into arrays.  It holds
none of the method's arithmetic (no LZW, no pooling, no logits): the CPU oracle
and the HIP path are both fed the arrays made here and share nothing else.

The arrays stand in for the paper's workloads (base-token IDs of code, math,
chat, multilingual and web text under 32K..150K-entry tokenizers; section 3
"Experiments", token-efficiency table): those corpora and tokenizers are not
available here, so token streams are Zipf-distributed IDs with planted repeats.
Shapes follow the five benchmark configurations.

bf16 tensors are handed around as uint16 bit patterns in numpy arrays.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Tuple

import numpy as np

# ---------------------------------------------------------------------------
# The five benchmark configurations.
#   mode "motif"    : copies of a small pool of seeded motifs are planted
#   mode "selfcopy" : copies of earlier spans of the same sequence are planted
#   copy_frac       : expected fraction of positions covered by a planted copy
# ---------------------------------------------------------------------------
CONFIGS: Dict[str, dict] = {
    "c1": dict(name="c1_tiny", B=2, N=512, V=32000, d=256, dtype="f32", M=3, cap=1024,
               zipf_s=1.1, copy_frac=0.20, span=(2, 6), mode="motif", pool="mean", seed=1000),
    "c2": dict(name="c2_prefill_llama3_8b", B=8, N=4096, V=128256, d=4096, dtype="bf16", M=3, cap=2048,
               zipf_s=1.1, copy_frac=0.30, span=(2, 8), mode="motif", pool="mean", seed=2000),
    "c3": dict(name="c3_decode_step", B=64, N=8192, V=128256, d=4096, dtype="bf16", M=3, cap=4096,
               zipf_s=1.1, copy_frac=0.20, span=(2, 6), mode="motif", pool="mean", seed=3000),
    "c4": dict(name="c4_long_code_like", B=4, N=32768, V=32064, d=3072, dtype="bf16", M=4, cap=8192,
               zipf_s=1.05, copy_frac=0.50, span=(4, 32), mode="selfcopy", pool="mean", seed=4000),
    "c5": dict(name="c5_large_vocab_deep_merges", B=16, N=16384, V=151936, d=3584, dtype="bf16", M=5,
               cap=16384, zipf_s=1.2, copy_frac=0.40, span=(2, 10), mode="motif", pool="weighted",
               seed=5000),
}

N_MOTIFS = 64          # size of the motif pool (a choice of this build)
_CHUNK_ELEMS = 1 << 24  # elements per independently seeded chunk of a big matrix


def scaled(cfg: dict, **over) -> dict:
    """A copy of a configuration with some sizes replaced (for small parity cases)."""
    out = dict(cfg)
    out.update(over)
    return out


# ---------------------------------------------------------------------------
# token streams
# ---------------------------------------------------------------------------
def _zipf_sampler(rng: np.random.Generator, V: int, s: float):
    """Return draw(n) -> int64 IDs with p(rank r) ~ r^-s, ranks scattered by a seeded permutation."""
    ranks = np.arange(1, V + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-s))
    cdf /= cdf[-1]
    perm = rng.permutation(V)

    def draw(n: int) -> np.ndarray:
        u = rng.random(n)
        r = np.searchsorted(cdf, u, side="left")
        np.minimum(r, V - 1, out=r)
        return perm[r]

    return draw


def make_tokens(cfg: dict) -> np.ndarray:
    """int32 [B, N] base-token IDs in [0, V)."""
    B, N, V = cfg["B"], cfg["N"], cfg["V"]
    lo, hi = cfg["span"]
    p = cfg["copy_frac"]
    rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 0))
    draw = _zipf_sampler(rng, V, cfg["zipf_s"])
    mean_len = 0.5 * (lo + hi)
    q = p / (p + (1.0 - p) * mean_len) if p > 0 else 0.0

    motifs = []
    if cfg["mode"] == "motif":
        lens = rng.integers(lo, hi + 1, size=N_MOTIFS)
        motifs = [draw(int(L)) for L in lens]

    out = np.empty((B, N), dtype=np.int32)
    for b in range(B):
        fill = draw(N)
        start = rng.random(N) < q
        pick = rng.integers(0, N_MOTIFS, size=N)
        span_len = rng.integers(lo, hi + 1, size=N)
        src_u = rng.random(N)
        x = out[b]
        i = 0
        while i < N:
            if start[i]:
                if cfg["mode"] == "motif":
                    m = motifs[int(pick[i])]
                    L = min(len(m), N - i)
                    x[i:i + L] = m[:L]
                    i += L
                    continue
                L = int(span_len[i])
                if i >= L:
                    j = int(src_u[i] * (i - L + 1))
                    L = min(L, N - i)
                    x[i:i + L] = x[j:j + L]
                    i += L
                    continue
            x[i] = fill[i]
            i += 1
    return out


def make_lens(cfg: dict, ragged: bool = False) -> np.ndarray:
    """int32 [B] valid lengths: all N, or (ragged) a seeded mix that includes 0, 1 and N."""
    B, N = cfg["B"], cfg["N"]
    if not ragged:
        return np.full(B, N, dtype=np.int32)
    rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 7))
    lens = rng.integers(0, N + 1, size=B).astype(np.int32)
    special = [N, 0, 1, max(N - 1, 0)]
    for k, v in enumerate(special[:B]):
        lens[k] = v
    return lens


# ---------------------------------------------------------------------------
# dense tensors
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (library conversion) and return the uint16 bit patterns."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def normal_matrix(seed: int, rows: int, cols: int, std: float, dtype: str, threads: int = 8) -> np.ndarray:
    """[rows, cols] N(0, std^2) samples, float32 (dtype 'f32') or bf16 bit patterns (dtype 'bf16').

    The matrix is cut into fixed row blocks, each with its own child seed, so the
    result does not depend on the number of threads used.
    """
    rows_per = max(1, _CHUNK_ELEMS // max(cols, 1))
    n_chunks = max(1, math.ceil(rows / rows_per))
    children = np.random.SeedSequence(seed).spawn(n_chunks)
    out = np.empty((rows, cols), dtype=np.float32 if dtype == "f32" else np.uint16)

    def work(c: int) -> None:
        r0 = c * rows_per
        r1 = min(rows, r0 + rows_per)
        g = np.random.Generator(np.random.PCG64(children[c]))
        blk = g.standard_normal((r1 - r0, cols), dtype=np.float32)
        blk *= np.float32(std)
        if dtype == "f32":
            out[r0:r1] = blk
        else:
            out[r0:r1] = f32_to_bf16_bits(blk)

    if n_chunks == 1 or threads <= 1:
        for c in range(n_chunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(n_chunks)))
    return out


def make_embeddings(cfg: dict) -> np.ndarray:
    """[V, d] base embedding / unembedding matrix, N(0, 0.02)."""
    return normal_matrix(cfg["seed"] + 1, cfg["V"], cfg["d"], 0.02, cfg["dtype"])


def make_hidden(cfg: dict, rows: int) -> np.ndarray:
    """[rows, d] hidden states, N(0, 1)."""
    return normal_matrix(cfg["seed"] + 2, rows, cfg["d"], 1.0, cfg["dtype"])


def make_pool_weights(cfg: dict) -> np.ndarray:
    """float32 [8] raw position weights (only the first M are used; zeros for mean pooling)."""
    w = np.zeros(8, dtype=np.float32)
    if cfg["pool"] == "weighted":
        rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 3))
        w[: cfg["M"]] = rng.standard_normal(cfg["M"]).astype(np.float32)
    return w


def make_encoder(cfg: dict, n_layers: int = 2, n_heads: int = 32, d_ff: int = 0, attention_only: bool = False,
                 with_pos: bool = True) -> dict:
    """Random-init parameters of a learned hyper-encoder (trained weights are not available here).

    Matrices [out, in] in the configuration's storage format, N(0, 1/in) (the projections behind the residual
    sum, w_o and w_2, N(0, 1/(4 in)) so that the residual stream keeps the scale of the embeddings' sum);
    biases N(0, 0.02), LayerNorm scales 1 + N(0, 0.1) and shifts N(0, 0.05), float32; slot positions [M, d]
    N(0, 0.02) like the embedding table.  d_ff = 0 means 4 d."""
    d, dtype, M = cfg["d"], cfg["dtype"], cfg["M"]
    d_ff = d_ff or 4 * d
    seed = cfg["seed"] + 100
    rng = np.random.Generator(np.random.PCG64(seed))

    def vec(n, mean, std):
        return (mean + std * rng.standard_normal(n)).astype(np.float32)

    layers = []
    for li in range(n_layers):
        s = seed + 10 * (li + 1)
        lay = dict(ln1_g=vec(d, 1.0, 0.1), ln1_b=vec(d, 0.0, 0.05),
                   w_qkv=normal_matrix(s + 1, 3 * d, d, d ** -0.5, dtype), b_qkv=vec(3 * d, 0.0, 0.02),
                   w_o=normal_matrix(s + 2, d, d, 0.5 * d ** -0.5, dtype), b_o=vec(d, 0.0, 0.02))
        if not attention_only:
            lay.update(ln2_g=vec(d, 1.0, 0.1), ln2_b=vec(d, 0.0, 0.05),
                       w_1=normal_matrix(s + 3, d_ff, d, d ** -0.5, dtype), b_1=vec(d_ff, 0.0, 0.02),
                       w_2=normal_matrix(s + 4, d, d_ff, 0.5 * d_ff ** -0.5, dtype), b_2=vec(d, 0.0, 0.02))
        layers.append(lay)
    pos = normal_matrix(seed + 5, M, d, 0.02, dtype) if with_pos else None
    return dict(n_heads=n_heads, attention_only=attention_only, d_ff=0 if attention_only else d_ff, pos=pos,
                layers=layers)


def make_step_codes(cfg: dict, sizes: np.ndarray, step: int) -> np.ndarray:
    """int32 [B] one new code per sequence for decode step `step`, uniform over the valid IDs
    [0, V + sizes[b]) with half of the draws forced into the hypertoken range when it is non-empty."""
    rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 4 + 17 * step))
    V = cfg["V"]
    sizes = np.asarray(sizes, dtype=np.int64)
    u = rng.random(sizes.shape[0])
    hyper = (rng.random(sizes.shape[0]) < 0.5) & (sizes > 0)
    base_draw = np.minimum((u * V).astype(np.int64), V - 1)
    hyper_draw = V + np.minimum((u * sizes).astype(np.int64), np.maximum(sizes - 1, 0))
    return np.where(hyper, hyper_draw, base_draw).astype(np.int32)


def sample_rows(cfg: dict, rows_per_seq: int, per_seq: int) -> np.ndarray:
    """Seeded sample of global row indices: `per_seq` rows of each sequence, first and last included."""
    rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 5))
    out = []
    for b in range(cfg["B"]):
        k = min(per_seq, rows_per_seq)
        if k >= rows_per_seq:
            loc = np.arange(rows_per_seq)
        else:
            inner = rng.choice(np.arange(1, rows_per_seq - 1), size=max(k - 2, 0), replace=False)
            loc = np.unique(np.concatenate([[0, rows_per_seq - 1], inner]))
        out.append(b * rows_per_seq + loc)
    return np.concatenate(out).astype(np.int64)
