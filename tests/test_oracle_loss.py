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


def _loss(H, Wb, Wh, C, t, g):
    nll = oracle.extended_nll(H, Wb, Wh, C, "f32", t)["nll"]
    ok = np.isfinite(nll)
    return float((g[ok] * nll[ok]).sum())


def test_backward_matches_central_differences_of_the_pinned_forward():
    """The forward oracle is pinned above; its central differences pin the gradient formulas (float32 storage
    means the step must change the stored value: steps are powers of two on O(1) inputs)."""
    rng = np.random.default_rng(5)
    rows, V, cap, C, d = 4, 9, 5, 3, 6
    H = rng.normal(size=(rows, d)).astype(np.float32)
    Wb = rng.normal(size=(V, d)).astype(np.float32)
    Wh = rng.normal(size=(cap, d)).astype(np.float32)
    t = np.array([2, V + 1, -1, V + C + 1])             # base target, hyper target, none, names no column
    g = np.array([1.0, 0.5, 3.0, 2.0])
    r = oracle.extended_nll_backward(H, Wb, Wh, C, "f32", t, g)
    eps = 2.0 ** -10
    for name, X, G in (("dH", H, r["dH"]), ("dW_base", Wb, r["dW_base"]), ("dW_hyper", Wh, r["dW_hyper"])):
        num = np.zeros_like(G)
        for idx in np.ndindex(X.shape):
            old = X[idx]
            X[idx] = old + np.float32(eps)
            up = _loss(H, Wb, Wh, C, t, g)
            X[idx] = old - np.float32(eps)
            dn = _loss(H, Wb, Wh, C, t, g)
            X[idx] = old
            num[idx] = (up - dn) / (2 * eps)
        assert np.allclose(G, num, rtol=0, atol=2e-5), name
    assert (r["dH"][2] == 0).all() and (r["dH"][3] == 0).all()      # rows without a usable target
    assert (r["dW_hyper"][C:] == 0).all()                           # slots that are not columns


def test_backward_matches_library_autograd():
    import torch

    rng = np.random.default_rng(6)
    rows, V, cap, C, d = 7, 20, 6, 4, 8
    H = rng.normal(size=(rows, d)).astype(np.float32)
    Wb = rng.normal(size=(V, d)).astype(np.float32)
    Wh = rng.normal(size=(cap, d)).astype(np.float32)
    t = rng.integers(0, V + C, size=rows)
    g = rng.uniform(0.5, 2.0, size=rows)
    r = oracle.extended_nll_backward(H, Wb, Wh, C, "f32", t, g)
    tH = torch.tensor(H, dtype=torch.float64, requires_grad=True)
    tWb = torch.tensor(Wb, dtype=torch.float64, requires_grad=True)
    tWh = torch.tensor(Wh, dtype=torch.float64, requires_grad=True)
    logits = tH @ torch.cat([tWb, tWh[:C]]).T
    loss = (torch.tensor(g) * torch.nn.functional.cross_entropy(logits, torch.tensor(t), reduction="none")).sum()
    loss.backward()
    assert np.allclose(r["dH"], tH.grad.numpy(), atol=1e-12)
    assert np.allclose(r["dW_base"], tWb.grad.numpy(), atol=1e-12)
    assert np.allclose(r["dW_hyper"], tWh.grad.numpy(), atol=1e-12)
    # each row of dZ sums to zero (softmax minus one-hot), so shifting every weight row by a vector leaves dH's
    # response unchanged: dZ @ (W + 1 c^T) = dZ @ W
    assert np.allclose(r["dZ"].sum(axis=1), 0, atol=1e-12)


def test_pooling_backward_is_the_transpose_of_the_pooling():
    """<dW, pool(E)> = <pool^T(dW), E> for random E and dW (the pooling is linear in E), mean and weighted."""
    rng = np.random.default_rng(7)
    V, d, cap = 11, 5, 6
    entries = [(1, 2), (3, 3, 4), (10,), (0, 9, 1)]
    for pool, w in (("mean", ()), ("weighted", (0.3, -1.0, 0.7))):
        E = rng.normal(size=(V, d)).astype(np.float32)
        dW = rng.normal(size=(cap, d))
        W = oracle.hyper_embed(E, "f32", entries, cap, pool, w).astype(np.float64)
        dE = oracle.hyper_embed_backward(dW, entries, V, pool, w)
        assert abs((dW * W).sum() - (dE * E.astype(np.float64)).sum()) < 1e-5
        assert (dE[[5, 6, 7, 8]] == 0).all()                        # tokens in no entry
    # a token that occurs twice in an entry receives the row twice
    dE = oracle.hyper_embed_backward(np.ones((1, d)), [(3, 3)], V)
    assert np.allclose(dE[3], 1.0)
