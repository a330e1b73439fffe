"""GPU parity: extended_nll_backward (gradient of the next-code objective of section 2.4 over the extended
vocabulary, into the hidden rows and both unembedding matrices) and hyper_embed_backward (through the pooling)
through the C ABI against the float64 oracle.

Bar.  The HIP path rounds the gradient with respect to the logits to bf16 once (relative 2^-9 per element) and
the results to bf16; the products accumulate in fp32.  An output element is a sum of many such terms with
independent rounding errors, so its error is far below 2^-9 of the sum of the terms' magnitudes; what is
asserted is |gpu - ref| <= 2e-2 * (largest |ref| of the output row) per element.  Rows of dH without a usable
target and rows of dW_hyper that are no columns are exactly zero.
"""
import numpy as np
import pytest

import oracle
from paper_2506_01084_amd import workloads as wl

from helpers import gpu_encode, oracle_encode_batch, storage_to_host, torch_storage
from test_gpu_nll import _targets_from_codes

pytestmark = pytest.mark.gpu


def _close(got_bits, ref, label):
    got = oracle.bf16_bits_to_f64(got_bits)
    scale = np.abs(ref).max(axis=-1, keepdims=True)
    bad = np.abs(got - ref) > 2e-2 * scale + 1e-30
    assert not bad.any(), f"{label}: {bad.sum()} elements off, worst {np.abs(got - ref).max():.3e} (scale {scale.max():.3e})"
    zero_rows = (scale[:, 0] == 0)
    assert (got[zero_rows] == 0).all(), f"{label}: rows that must be zero"


def _setup(cfg, lens):
    import torch
    from paper_2506_01084_amd import api

    B, N, V, cap, d = cfg["B"], cfg["N"], cfg["V"], cfg["cap"], cfg["d"]
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    H = wl.make_hidden(cfg, B * N)
    w = wl.make_pool_weights(cfg)
    ctx = api.Context(B=B, V=V, M=cfg["M"], cap=cap, d=d, dtype="bf16", pool=cfg["pool"], w=w.tolist())
    gpu_encode(ctx, tokens, lens)
    ref = oracle_encode_batch(tokens, lens, V, cfg["M"], cap)
    rng = np.random.default_rng(cfg["seed"] + 9)
    targets = _targets_from_codes(ref, B, N, V, rng)
    grad = rng.uniform(0.25, 2.0, size=B * N).astype(np.float32)
    d_E = torch_storage(E, "bf16")
    d_W = torch.zeros((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.hyper_embed(d_E, d_W)
    d_H = torch_storage(H, "bf16")
    d_t = torch.from_numpy(targets.reshape(-1)).cuda()
    nll = torch.empty(B * N, dtype=torch.float32, device="cuda")
    lse = torch.empty(B * N, dtype=torch.float32, device="cuda")
    ctx.extended_nll(d_H, N, d_E, d_W, d_t, nll, lse)
    torch.cuda.synchronize()
    return ctx, ref, E, H, w, targets, grad, d_E, d_W, d_H, d_t, lse


@pytest.mark.parametrize("chunk", [0, 1, 2])          # sequences per pass of the backward (0: all at once)
@pytest.mark.parametrize("B,N,V,d,M,cap,pool,use_grad", [
    (3, 150, 500, 64, 3, 64, "mean", True),
    (2, 300, 700, 128, 4, 200, "weighted", False),
    (5, 333, 1000, 192, 3, 100, "mean", True),          # ragged tiles in every product
    (1, 700, 2100, 256, 3, 300, "mean", True),          # several row tiles per sequence
])
def test_gradients_match_oracle(B, N, V, d, M, cap, pool, use_grad, chunk):
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, d=d, M=M, cap=cap, pool=pool, zipf_s=1.3, seed=13 * B + d)
    print(f"[case] nll backward B={B} N={N} V={V} d={d} cap={cap}", flush=True)
    lens = wl.make_lens(cfg, ragged=True)
    ctx, ref, E, H, w, targets, grad, d_E, d_W, d_H, d_t, lse = _setup(cfg, lens)
    d_g = torch.from_numpy(grad).cuda() if use_grad else None
    dH = torch.full((B * N, d), 9.0, dtype=torch.bfloat16, device="cuda")
    dWb = torch.full((V, d), 9.0, dtype=torch.bfloat16, device="cuda")
    dWh = torch.full((B, cap, d), 9.0, dtype=torch.bfloat16, device="cuda")
    ctx.set_option(api.OPT_BACKWARD_CHUNK, chunk)      # dW_base of a later chunk adds to the earlier ones' bf16 sum
    ctx.extended_nll_backward(d_H, N, d_E, d_W, d_t, lse, d_g, dH, dWb, dWh)
    dE = torch.zeros((V, d), dtype=torch.float32, device="cuda")
    ctx.hyper_embed_backward(dWh, dE)
    torch.cuda.synchronize()
    dH_h, dWb_h, dWh_h = (storage_to_host(t, "bf16") for t in (dH, dWb, dWh))
    want_dWb = np.zeros((V, d))
    want_dE = np.zeros((V, d))
    W_host = storage_to_host(d_W, "bf16")
    for b in range(B):
        sl = slice(b * N, (b + 1) * N)
        g = grad[sl] if use_grad else np.ones(N)
        r = oracle.extended_nll_backward(H[sl], E, W_host[b], len(ref[b][1]), "bf16", targets[b], g)
        _close(dH_h[sl], r["dH"], f"dH seq {b}")
        _close(dWh_h[b], r["dW_hyper"], f"dW_hyper seq {b}")
        want_dWb += r["dW_base"]
        # the pooling's backward is checked on what it was given: the GPU's own (rounded) dW_hyper
        want_dE += oracle.hyper_embed_backward(oracle.bf16_bits_to_f64(dWh_h[b]), ref[b][1], V, pool, w)
    _close(dWb_h, want_dWb, "dW_base")
    got_dE = dE.cpu().numpy().astype(np.float64)
    scale = np.abs(want_dE).max(axis=1, keepdims=True)
    assert (np.abs(got_dE - want_dE) <= 1e-4 * scale + 1e-30).all(), "dE (fp32 sums of bf16 rows)"
    assert (got_dE[scale[:, 0] == 0] == 0).all()
    ctx.close()


def test_full_size_c2_sampled_rows():
    """Configuration 2 (32768 rows x 130304 columns): sampled rows of dH, of dW_base and of dW_hyper."""
    import time
    import torch

    cfg = wl.CONFIGS["c2"]
    B, N, V, cap, d = cfg["B"], cfg["N"], cfg["V"], cfg["cap"], cfg["d"]
    t0 = time.time()
    print("[case] full size nll backward c2", flush=True)
    ctx, ref, E, H, w, targets, grad, d_E, d_W, d_H, d_t, lse = _setup(cfg, np.full(B, N, dtype=np.int32))
    d_g = torch.from_numpy(grad).cuda()
    dH = torch.empty((B * N, d), dtype=torch.bfloat16, device="cuda")
    dWb = torch.empty((V, d), dtype=torch.bfloat16, device="cuda")
    dWh = torch.empty((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.extended_nll_backward(d_H, N, d_E, d_W, d_t, lse, d_g, dH, dWb, dWh)
    torch.cuda.synchronize()
    print(f"  GPU done {time.time() - t0:.1f}s", flush=True)
    W_host = storage_to_host(d_W, "bf16")
    # dH of a few rows: one row of the oracle at a time
    dH_h = storage_to_host(dH, "bf16")
    for b, i in ((0, 0), (3, 1234), (7, N - 1)):
        r = oracle.extended_nll_backward(H[b * N + i:b * N + i + 1], E, W_host[b], len(ref[b][1]), "bf16",
                                         targets[b, i:i + 1], grad[b * N + i:b * N + i + 1])
        _close(dH_h[b * N + i:b * N + i + 1], r["dH"], f"dH row ({b}, {i})")
    print(f"  dH rows checked {time.time() - t0:.1f}s", flush=True)
    # dW rows need dZ[:, v] of every hidden row: the oracle computes the logits of a few columns only, with the
    # row statistics (lse) taken from the GPU's forward pass, which its own test pins
    lse_h = lse.cpu().numpy().astype(np.float64)
    H64 = oracle.bf16_bits_to_f64(H)
    g64 = grad.astype(np.float64)
    tflat = targets.reshape(-1)
    usable = np.zeros(B * N, dtype=bool)
    for b in range(B):
        tb = targets[b]
        usable[b * N:(b + 1) * N] = (tb >= 0) & (tb < V + len(ref[b][1]))
    geff = np.where(usable, g64, 0.0)
    dWb_h = storage_to_host(dWb, "bf16")
    for v in (0, 777, V - 1, int(tflat[5]) if 0 <= tflat[5] < V else 11):
        z = H64 @ oracle.bf16_bits_to_f64(E[v])
        dz = geff * (np.exp(z - lse_h) - (tflat == v))
        _close(dWb_h[v:v + 1], (dz @ H64)[None, :], f"dW_base row {v}")
    dWh_h = storage_to_host(dWh, "bf16")
    for b, e in ((0, 0), (5, 2047)):
        sl = slice(b * N, (b + 1) * N)
        z = H64[sl] @ oracle.bf16_bits_to_f64(W_host[b, e])
        dz = geff[sl] * (np.exp(z - lse_h[sl]) - (tflat[sl] == V + e))
        _close(dWh_h[b, e:e + 1], (dz @ H64[sl])[None, :], f"dW_hyper ({b}, {e})")
    print(f"  dW rows checked {time.time() - t0:.1f}s", flush=True)
    ctx.close()


def test_edge_cases_no_hypertokens_no_targets_and_odd_row_counts():
    import torch
    from paper_2506_01084_amd import api

    # cap = 0: base vocabulary only; 77 rows per sequence (not a multiple of 64), V not a multiple of 64
    B, N, V, d = 3, 77, 333, 64
    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, d=d, M=3, cap=0, seed=31)
    E = wl.make_embeddings(cfg)
    H = wl.make_hidden(cfg, B * N)
    rng = np.random.default_rng(2)
    targets = rng.integers(0, V, size=(B, N)).astype(np.int32)
    targets[1] = -1                                            # a sequence without any target
    targets[2, ::2] = V + 5                                    # names no column
    ctx = api.Context(B=B, V=V, M=3, cap=0, d=d, dtype="bf16")
    ctx.reset()
    d_E, d_H = torch_storage(E, "bf16"), torch_storage(H, "bf16")
    d_W = torch.zeros((B, 0, d), dtype=torch.bfloat16, device="cuda")
    d_t = torch.from_numpy(targets.reshape(-1)).cuda()
    nll = torch.empty(B * N, dtype=torch.float32, device="cuda")
    lse = torch.empty_like(nll)
    ctx.extended_nll(d_H, N, d_E, d_W, d_t, nll, lse)
    dH = torch.full((B * N, d), 9.0, dtype=torch.bfloat16, device="cuda")
    dWb = torch.full((V, d), 9.0, dtype=torch.bfloat16, device="cuda")
    dWh = torch.zeros((B, 0, d), dtype=torch.bfloat16, device="cuda")
    for rep in range(2):                                       # the second call reuses the work space
        ctx.extended_nll_backward(d_H, N, d_E, d_W, d_t, lse, None, dH, dWb, dWh)
    dE = torch.zeros((V, d), dtype=torch.float32, device="cuda")
    ctx.hyper_embed_backward(dWh, dE)
    torch.cuda.synchronize()
    assert (dE == 0).all()
    dH_h, dWb_h = storage_to_host(dH, "bf16"), storage_to_host(dWb, "bf16")
    want_dWb = np.zeros((V, d))
    for b in range(B):
        sl = slice(b * N, (b + 1) * N)
        r = oracle.extended_nll_backward(H[sl], E, np.zeros((0, d), dtype=np.uint16), 0, "bf16", targets[b], np.ones(N))
        _close(dH_h[sl], r["dH"], f"dH seq {b}")
        want_dWb += r["dW_base"]
    _close(dWb_h, want_dWb, "dW_base")
    assert (oracle.bf16_bits_to_f64(dH_h[N:2 * N]) == 0).all()
    ctx.close()

    # fp32 contexts are refused, not silently served by something else
    ctx = api.Context(B=1, V=100, M=3, cap=8, d=64, dtype="f32")
    ctx.reset()
    z = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda")
    with pytest.raises(api.Z2ZError):
        ctx.extended_nll_backward(z(4, 64), 4, z(100, 64), z(1, 8, 64), torch.zeros(4, dtype=torch.int32, device="cuda"),
                                  z(4), None, z(4, 64), z(100, 64), z(1, 8, 64))
    ctx.close()
