"""Pins for the sampling oracle (CPU only): the generator against published known-answer vectors, the
Gumbel-max draw against the distribution it must follow, and the limits that reduce to argmax."""
import os

import numpy as np

from oracle import sampling
from oracle.sampling import philox4x32_10, sample_row, uniforms


def test_philox_known_answers(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        out = philox4x32_10(w[0:4], (w[4], w[5]))
        assert [int(x) for x in out] == w[6:10]
        n += 1
    assert n == 3


def test_philox_vectorised_equals_scalar_and_is_injective_on_counters():
    ctr = np.zeros((4096, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(4096)
    ctr[:, 1] = 7
    out = philox4x32_10(ctr, (123, 456))
    for i in (0, 1, 17, 4095):
        assert (out[i] == philox4x32_10([i, 7, 0, 0], (123, 456))).all()
    # a bijection of the counter for a fixed key: distinct counters give distinct 128-bit outputs
    assert len({tuple(int(x) for x in row) for row in out}) == 4096


def test_uniforms_layout_and_range():
    u = uniforms(seed=(5 << 32) | 9, step=(3 << 32) | 11, row=2, n_cols=10)
    w = philox4x32_10([[0, 2, 11, 3], [1, 2, 11, 3], [2, 2, 11, 3]], (9, 5)).reshape(-1)[:10]
    assert (u == ((w >> 9).astype(np.float64) + 0.5) / 2 ** 23).all()
    big = uniforms(1, 2, 3, 100000)
    assert big.min() > 0.0 and big.max() < 1.0
    assert abs(big.mean() - 0.5) < 5e-3 and abs(big.var() - 1 / 12) < 2e-3
    assert (big.astype(np.float32).astype(np.float64) == big).all()        # exactly representable in float32


def test_draws_follow_softmax_of_scaled_logits():
    """Chi-square of 20000 draws (one per step) against softmax(l / T) on a 9-column row."""
    logits = np.array([2.0, 0.5, -1.0, 1.5, 0.0, 3.0, -2.5, 1.0, 0.25])
    for T, seed in ((1.0, 11), (0.5, 12), (2.0, 13)):
        p = np.exp(logits / T - (logits / T).max())
        p /= p.sum()
        n = 20000
        counts = np.zeros(9)
        lp = {}
        for step in range(n):
            r = sample_row(logits, T, seed, step, row=3)
            counts[r["token"]] += 1
            lp[r["token"]] = r["logprob"]
        chi2 = ((counts - n * p) ** 2 / (n * p)).sum()
        assert chi2 < 27.9, (T, chi2)                                      # 99.95 % point of chi-square(8)
        for v, l in lp.items():
            assert abs(l - np.log(p[v])) < 1e-12                           # the reported log-probability


def test_limits_and_invariances():
    rng = np.random.default_rng(0)
    logits = rng.normal(size=50)
    am = int(np.argmax(logits))
    for step in range(20):
        cold = sample_row(logits, 1e-4, 1, step, 0)                        # T -> 0: the argmax, probability 1
        assert cold["token"] == am and abs(cold["logprob"]) < 1e-9
        a = sample_row(logits, 0.7, 1, step, 0)
        b = sample_row(logits + 123.0, 0.7, 1, step, 0)                    # a shift of all logits changes nothing
        assert a["token"] == b["token"] and abs(a["logprob"] - b["logprob"]) < 1e-9
        assert a["gap"] >= 0.0
    # different rows, steps and seeds draw different numbers
    base = uniforms(1, 0, 0, 64)
    assert not (base == uniforms(1, 0, 1, 64)).any()
    assert not (base == uniforms(1, 1, 0, 64)).any()
    assert not (base == uniforms(2, 0, 0, 64)).any()


def test_extended_sample_never_picks_a_missing_column():
    rng = np.random.default_rng(5)
    V, cap, C, d = 40, 8, 3, 16
    H = rng.normal(size=(4, d)).astype(np.float32)
    Wb = rng.normal(size=(V, d)).astype(np.float32)
    Wh = rng.normal(size=(cap, d)).astype(np.float32) * 50.0               # huge rows beyond C must stay invisible
    for step in range(50):
        r = sampling.extended_sample(H, Wb, Wh, C, "f32", 1.0, 99, step, row0=8)
        assert (r["token"] < V + C).all() and (r["logprob"] <= 0).all()
        assert r["logits"].shape[1] == V + C
