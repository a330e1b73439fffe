"""Pins for the negative-log-likelihood oracle (CPU only)."""
import numpy as np
from scipy.special import log_softmax

import oracle


def _case(seed=0, rows=5, V=30, cap=8, C=5, d=12):
    rng = np.random.default_rng(seed)
    H = rng.normal(size=(rows, d)).astype(np.float32)
    Wb = rng.normal(size=(V, d)).astype(np.float32)
    Wh = rng.normal(size=(cap, d)).astype(np.float32)
    return H, Wb, Wh, C


def test_equals_library_log_softmax_and_normalises():
    H, Wb, Wh, C = _case()
    V = Wb.shape[0]
    W = np.concatenate([Wb, Wh[:C]]).astype(np.float64)
    ref = -log_softmax(H.astype(np.float64) @ W.T, axis=1)          # library routine on the plain definition
    total = np.zeros(H.shape[0])
    for t in range(V + C):
        r = oracle.extended_nll(H, Wb, Wh, C, "f32", np.full(H.shape[0], t))
        assert np.allclose(r["nll"], ref[:, t], rtol=0, atol=1e-12)
        assert (r["nll"] >= 0).all()
        total += np.exp(-r["nll"])
    assert np.allclose(total, 1.0, atol=1e-12)                      # the probabilities of all targets sum to one


def test_ignored_missing_and_hyper_targets():
    H, Wb, Wh, C = _case(seed=3)
    V = Wb.shape[0]
    t = np.array([-1, V + C, V + C - 1, 0, V + 7])
    r = oracle.extended_nll(H, Wb, Wh, C, "f32", t)
    assert r["nll"][0] == 0.0                                       # no target
    assert np.isinf(r["nll"][1]) and np.isinf(r["nll"][4])          # names no existing column
    assert np.isfinite(r["nll"][2]) and np.isfinite(r["nll"][3])
    # a hyper row equal to a base row gets the same likelihood as that base token
    Wh2 = Wh.copy()
    Wh2[2] = Wb[4]
    a = oracle.extended_nll(H, Wb, Wh2, C, "f32", np.full(5, V + 2))["nll"]
    b = oracle.extended_nll(H, Wb, Wh2, C, "f32", np.full(5, 4))["nll"]
    assert np.allclose(a, b, atol=1e-12)
    # with H = 0 every column is equally likely
    z = oracle.extended_nll(np.zeros_like(H), Wb, Wh, C, "f32", np.arange(5))["nll"]
    assert np.allclose(z, np.log(V + C))
