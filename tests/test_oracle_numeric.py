"""Pins for the pooling and logit oracles and for the bf16 conversions they rely on."""
import math
import random
from fractions import Fraction

import numpy as np
import pytest

from oracle import (bf16_bits_to_f64, extended_logits, f64_to_bf16_bits, hyper_embed, lzw_encode,
                    pool_coefficients)


# ---------------------------------------------------------------------------
# bf16 <-> float64: checked against exact rational arithmetic
# ---------------------------------------------------------------------------
def _bf16_neighbours(x: float):
    """The two bf16 values around a positive normal x, as exact Fractions (8-bit significand)."""
    m, e = math.frexp(x)                 # x = m * 2^e, 0.5 <= m < 1
    ulp = Fraction(2) ** (e - 8)
    lo = (Fraction(x) // ulp) * ulp
    return lo, lo + ulp, ulp


def test_bf16_widening_is_exact():
    bits = np.array([0x0000, 0x3F80, 0xBF80, 0x3C00, 0x4049, 0x0080, 0x7F7F], dtype=np.uint16)
    want = [0.0, 1.0, -1.0, 2.0 ** -7, 3.140625, 2.0 ** -126, (2 - 2 ** -7) * 2.0 ** 127]
    assert bf16_bits_to_f64(bits).tolist() == want


def test_bf16_rounding_matches_exact_nearest_even():
    rnd = random.Random(11)
    xs = []
    for _ in range(3000):
        xs.append(rnd.uniform(-4, 4) * 10 ** rnd.uniform(-6, 3))
    # exact ties and near-ties, where two nearest roundings in a row go wrong
    for k in range(200):
        base = 1.0 + k / 128.0                      # a bf16 value in [1, 2.6)
        tie = base + 2.0 ** -8                      # halfway to the next bf16 value
        xs += [tie, tie + 2.0 ** -40, tie - 2.0 ** -40, tie + 2.0 ** -25, tie - 2.0 ** -25]
    xs = [x for x in xs if x != 0.0]
    got = bf16_bits_to_f64(f64_to_bf16_bits(np.array(xs)))
    for x, g in zip(xs, got):
        lo, hi, ulp = _bf16_neighbours(abs(x))
        fx = Fraction(abs(x))
        if fx - lo < hi - fx:
            want = lo
        elif fx - lo > hi - fx:
            want = hi
        else:                                       # tie -> even multiple of ulp
            want = lo if (lo / ulp) % 2 == 0 else hi
        assert Fraction(abs(float(g))) == want, x
        assert math.copysign(1, g) == math.copysign(1, x)
    # values already representable come back unchanged
    b = np.arange(0x3800, 0x4800, dtype=np.uint16)
    assert (f64_to_bf16_bits(bf16_bits_to_f64(b)) == b).all()


# ---------------------------------------------------------------------------
# P8: pooling closed forms
# ---------------------------------------------------------------------------
def test_pool_coefficients():
    assert pool_coefficients(3, "mean", []).tolist() == [1 / 3, 1 / 3, 1 / 3]
    a = pool_coefficients(2, "weighted", [0.0, math.log(3.0), 5.0])
    assert np.allclose(a, [0.25, 0.75], rtol=0, atol=1e-15)      # later raw weights do not enter
    a = pool_coefficients(4, "weighted", [0.3] * 8)
    assert np.allclose(a, 0.25, rtol=0, atol=1e-15)              # equal raw weights == mean


def test_mean_pool_closed_forms():
    rng = np.random.default_rng(0)
    V, d, M, cap = 12, 16, 4, 8
    E = rng.standard_normal((V, d)).astype(np.float32)
    entries = [(1, 2), (3, 3, 3), (0, 5, 7, 9), (4, 4)]
    W = hyper_embed(E, "f32", entries, cap, "mean")
    assert W.shape == (cap, d) and W.dtype == np.float32
    # the definition, retyped independently with float64 numpy
    for i, e in enumerate(entries):
        want = np.mean(np.stack([E[t].astype(np.float64) for t in e]), axis=0)
        assert np.allclose(W[i], want, rtol=1e-7, atol=0)
    # all-equal constituents: the mean is that row exactly (divisor is L, not M)
    assert (W[1] == E[3]).all() and (W[3] == E[4]).all()
    # rows beyond the codebook are zero
    assert (W[len(entries):] == 0).all()
    # one-hot embeddings: the result is the normalised histogram of the entry's tokens
    I = np.eye(V, dtype=np.float32)
    Wh = hyper_embed(I, "f32", [(2, 2, 5)], 1, "mean")
    want = np.zeros(V); want[2] = 2 / 3; want[5] = 1 / 3
    assert np.allclose(Wh[0], want, atol=1e-7)
    # divisor L vs M: a length-2 entry at M=4 has coefficients 1/2, which sum to one
    assert abs(Wh[0].sum() - 1.0) < 1e-6


def test_weighted_pool_reduces_to_mean_and_bf16_rounds_once():
    rng = np.random.default_rng(1)
    V, d = 9, 32
    from oracle import f64_to_bf16_bits as rnd_bf16
    Ebits = rnd_bf16(rng.standard_normal((V, d)) * 0.02)
    entries = [(0, 1), (2, 3, 4), (5, 6, 7, 8, 0)]
    Wm = hyper_embed(Ebits, "bf16", entries, 4, "mean")
    Ww = hyper_embed(Ebits, "bf16", entries, 4, "weighted", [0.0] * 8)
    assert Wm.dtype == np.uint16 and (Wm == Ww).all()
    # the stored value is the single nearest-even rounding of the exact mean
    Ed = bf16_bits_to_f64(Ebits)
    for i, e in enumerate(entries):
        exact = sum(Ed[t] for t in e) / len(e)
        assert (Wm[i] == rnd_bf16(exact)).all()
    # a weighted case by hand: w = (0, ln 3) -> 1/4, 3/4
    Ww = hyper_embed(Ebits, "bf16", [(1, 2)], 1, "weighted", [0.0, math.log(3.0)])
    assert (Ww[0] == rnd_bf16(0.25 * Ed[1] + 0.75 * Ed[2])).all()


# ---------------------------------------------------------------------------
# P9 / P10: logits
# ---------------------------------------------------------------------------
def _setup(seed, V=40, d=24, rows=7, cap=16, M=3, pool="mean", w=()):
    rng = np.random.default_rng(seed)
    E = (rng.standard_normal((V, d)) * 0.5).astype(np.float32)
    H = rng.standard_normal((rows, d)).astype(np.float32)
    toks = rng.integers(0, 5, size=60).tolist()
    _, entries, _ = lzw_encode(toks, V, M, cap)
    return E, H, entries


def test_logits_base_part_is_the_library_product_and_shapes():
    E, H, entries = _setup(2)
    cap = 16
    Wh = hyper_embed(E, "f32", entries, cap, "mean")
    out = extended_logits(H, E, Wh, len(entries), "f32")
    V = E.shape[0]
    assert out["logits"].shape == (H.shape[0], V + len(entries))
    ref = H.astype(np.float64) @ E.astype(np.float64).T
    assert np.allclose(out["logits"][:, :V], ref, rtol=1e-13, atol=1e-13)
    # transposed-operand mistake would fail this: element (r, v) by an explicit loop
    r, v = 3, 17
    s = sum(float(H[r, k]) * float(E[v, k]) for k in range(E.shape[1]))
    assert abs(out["logits"][r, v] - s) < 1e-12


@pytest.mark.parametrize("pool,w", [("mean", ()), ("weighted", (0.3, -1.0, 0.7, 0.0, 0.0))])
def test_hyper_logit_is_pooled_base_logit(pool, w):
    """Linearity: with exact (unrounded) pooling the hyper logit is the same pooling of the base logits."""
    E, H, entries = _setup(3)
    assert any(len(e) == 3 for e in entries) and any(len(e) == 2 for e in entries)
    V, cap = E.shape[0], 16
    Ed = E.astype(np.float64)
    Wexact = np.zeros((cap, E.shape[1]))
    for i, e in enumerate(entries):
        a = pool_coefficients(len(e), pool, w)
        Wexact[i] = sum(a[j] * Ed[t] for j, t in enumerate(e))
    # feed the exact rows as float64-representable "f32" only after checking the rounding gap is tiny
    Wh = hyper_embed(E, "f32", entries, cap, pool, w)
    out = extended_logits(H, E, Wh, len(entries), "f32")
    base = out["logits"][:, :V]
    for i, e in enumerate(entries):
        a = pool_coefficients(len(e), pool, w)
        want = sum(a[j] * base[:, t] for j, t in enumerate(e))
        assert np.allclose(out["logits"][:, V + i], want, rtol=0, atol=2e-6)   # float32 rounding of W_hyper


def test_lse_bounds_zero_hidden_and_masking():
    E, H, entries = _setup(4)
    V, cap = E.shape[0], 16
    Wh = hyper_embed(E, "f32", entries, cap, "mean")
    C = len(entries)
    out = extended_logits(H, E, Wh, C, "f32")
    assert (out["lse"] >= out["max"]).all()
    assert (out["lse"] <= out["max"] + math.log(V + C) + 1e-12).all()
    assert (out["argmax"] == out["logits"].argmax(axis=1)).all()
    assert np.allclose(out["max"], out["logits"][np.arange(len(H)), out["argmax"]])
    # softmax sums to one through the returned lse
    p = np.exp(out["logits"] - out["lse"][:, None])
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-12)
    # H = 0: all logits 0, lse = ln(V + C), argmax = lowest index
    z = extended_logits(np.zeros_like(H), E, Wh, C, "f32")
    assert (z["logits"] == 0).all() and (z["argmax"] == 0).all()
    assert np.allclose(z["lse"], math.log(V + C), atol=1e-12)
    # slots beyond C never appear: poison them and nothing changes
    Wp = Wh.copy(); Wp[C:] = 1e6
    o2 = extended_logits(H, E, Wp, C, "f32")
    assert (o2["logits"] == out["logits"]).all() and (o2["argmax"] == out["argmax"]).all()
    # fewer entries -> fewer columns
    o3 = extended_logits(H, E, Wh, 0, "f32")
    assert o3["logits"].shape[1] == V
    # margin is the top-1 minus top-2 gap
    srt = np.sort(out["logits"], axis=1)
    assert np.allclose(out["margin"], srt[:, -1] - srt[:, -2])


def test_logits_bf16_inputs_are_widened_exactly():
    rng = np.random.default_rng(5)
    V, d, rows = 30, 16, 4
    Eb = f64_to_bf16_bits(rng.standard_normal((V, d)) * 0.02)
    Hb = f64_to_bf16_bits(rng.standard_normal((rows, d)))
    Wh = hyper_embed(Eb, "bf16", [(1, 2), (1, 2, 3)], 2, "mean")
    out = extended_logits(Hb, Eb, Wh, 2, "bf16")
    ref = bf16_bits_to_f64(Hb) @ np.vstack([bf16_bits_to_f64(Eb), bf16_bits_to_f64(Wh)]).T
    assert np.allclose(out["logits"], ref, rtol=1e-14, atol=1e-14)
    # after the bf16 rounding of W_hyper, linearity holds to about 2^-8 of the logit scale
    base = out["logits"][:, :V]
    want = (base[:, 1] + base[:, 2]) / 2
    scale = np.abs(bf16_bits_to_f64(Hb)).sum(axis=1) * 0.02 * 3
    assert (np.abs(out["logits"][:, V] - want) <= scale * 2.0 ** -8).all()
