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


# ---- truncation (top-k / nucleus) ----------------------------------------------------------------------
def _brute_kept(z, k, p):
    """The rule spelled out with Python sorting and a running sum."""
    cols = sorted(range(len(z)), key=lambda v: (-z[v], v))
    q = np.exp(z - z.max())
    q = q / q.sum()
    n_p, acc = len(cols), 0.0
    if p < 1.0:
        for i, v in enumerate(cols):
            acc += q[v]
            if acc >= p:
                n_p = i + 1
                break
    n_k = len(cols) if k <= 0 else min(k, len(cols))
    return cols[:max(1, min(n_k, n_p))]


def test_kept_prefix_against_brute_force_and_ties():
    rng = np.random.default_rng(2)
    for trial in range(200):
        n = int(rng.integers(1, 12))
        z = np.round(rng.normal(size=n) * 2) / 2            # many exact ties
        k = int(rng.integers(0, n + 2))
        p = float(rng.choice([0.05, 0.3, 0.62, 0.9, 0.999, 1.0]))
        got = sampling.kept_prefix(z, k, p)
        assert got["kept"].tolist() == _brute_kept(z, k, p), (z, k, p)
        assert got["n"] == len(got["kept"]) >= 1


def test_truncated_draws_limits():
    rng = np.random.default_rng(4)
    logits = rng.normal(size=40) * 2
    am = int(np.argmax(logits))
    for step in range(30):
        full = sample_row(logits, 0.9, 3, step, 1)
        same = sampling.sample_row_truncated(logits, 0.9, 0, 1.0, 3, step, 1)             # both filters off
        assert same["token"] == full["token"] and abs(same["logprob"] - full["logprob"]) < 1e-12
        assert sampling.sample_row_truncated(logits, 0.9, 1, 1.0, 3, step, 1)["token"] == am      # k = 1
        assert sampling.sample_row_truncated(logits, 0.9, 0, 1e-9, 3, step, 1)["token"] == am     # p -> 0
        r = sampling.sample_row_truncated(logits, 0.9, 5, 0.8, 3, step, 1)
        assert r["token"] in r["kept"] and r["n_kept"] <= 5 and r["logprob"] <= 0


def test_truncated_draws_follow_the_renormalised_distribution():
    logits = np.array([2.0, 0.5, -1.0, 1.5, 0.0, 3.0, -2.5, 1.0, 0.25, 2.9])
    T, k, p = 1.3, 6, 0.85
    z = logits / T
    kept = sampling.kept_prefix(z, k, p)["kept"]
    q = np.exp(z[kept] - z[kept].max())
    q /= q.sum()
    n = 20000
    counts = dict.fromkeys(kept.tolist(), 0)
    for step in range(n):
        r = sampling.sample_row_truncated(logits, T, k, p, 21, step, 0)
        counts[r["token"]] += 1                              # a KeyError here would be a draw outside the kept set
        assert abs(r["logprob"] - np.log(q[kept.tolist().index(r["token"])])) < 1e-12
    c = np.array([counts[v] for v in kept.tolist()])
    chi2 = ((c - n * q) ** 2 / (n * q)).sum()
    assert chi2 < 30.0, chi2                                 # far beyond the 99.9 % point for <= 5 degrees of freedom
