"""GPU parity: hyper_encode_backward (the gradient of the learned hyper-encoder, for training f_phi with the
loss over the compressed sequence, section 2.4) through the C ABI against the float64 oracle.

Bar.  The HIP path runs forward and backward with bf16 rows between kernels (fp32 sums; the forward's residual
stream is fp32); the oracle
differentiates in float64 at the unrounded forward values.  A gradient tensor is a sum over all slot rows of
the call, so what is compared is each tensor as a whole: |got - want| <= TOL * max|want| per element.  Every
rounding on the way (about 6 per layer forward and 8 per layer backward, each a relative 2^-9 of a row element)
perturbs a row's contribution by a fraction of a percent; with two layers, 28 roundings all pushing one way
would be 28 * 2^-9 = 5.5e-2, independent ones add in quadrature (about 1e-2: the largest seen in the cases
below is 1.1e-2, over 3200 random shapes with up to three layers 2.4e-2 with a bf16 residual stream in the
forward pass, 1.5e-2 over 616 random shapes with the fp32 one).  TOL = 6e-2; the mean error over a
tensor has to stay below a tenth of that (seen: 2e-3 here, 4.4e-3 over the random shapes).
"""
import numpy as np
import pytest

import oracle
from paper_2506_01084_amd import workloads as wl

from helpers import encoder_to_device, gpu_encode, oracle_encode_batch, storage_to_host, torch_storage

pytestmark = pytest.mark.gpu

TOL = 6e-2


def _grad_buffers(enc, dtype="bf16"):
    """An encoder of the same shape whose tensors (filled with junk) receive the gradients."""
    junk = dict(n_heads=enc["n_heads"], attention_only=enc["attention_only"], d_ff=enc["d_ff"],
                pos=None if enc["pos"] is None else np.full_like(enc["pos"], 0x4123),
                layers=[{k: (np.full_like(v, 0x4123) if k.startswith("w_") else np.full_like(v, 9.0))
                         for k, v in lay.items()} for lay in enc["layers"]])
    return encoder_to_device(junk, dtype)


def _check(name, got, want, worst):
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == want.shape, name
    scale = max(np.abs(want).max(), 1e-30)
    err = np.abs(got - want) / scale
    worst[name] = (float(err.max()), float(err.mean()))
    assert np.isfinite(got).all(), name
    assert err.max() <= TOL, f"{name}: max error {err.max():.4f} of the tensor's largest gradient"
    assert err.mean() <= TOL / 10, f"{name}: mean error {err.mean():.4f}"


def _run_case(B, N, V, d, M, cap, n_layers, n_heads, d_ff, attn_only, with_pos, seed, seqs=None, lens_zero=True):
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=seed)
    lens = wl.make_lens(cfg, ragged=True)
    if B > 1 and lens_zero:
        lens[1] = 0
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype="bf16")
    gpu_encode(ctx, tokens, lens)
    ref = oracle_encode_batch(tokens, lens, V, M, cap)
    d_E = torch_storage(E, "bf16")
    enc = wl.make_encoder(cfg, n_layers=n_layers, n_heads=n_heads, d_ff=d_ff, attention_only=attn_only,
                          with_pos=with_pos)
    d_enc = encoder_to_device(enc, "bf16")
    d_grad = _grad_buffers(enc)
    dW = wl.normal_matrix(seed + 1, B * cap, d, 1.0, "bf16").reshape(B, cap, d)
    d_dW = torch_storage(dW, "bf16")
    dE = torch.zeros((V, d), dtype=torch.float32, device="cuda")
    ctx.hyper_encode_backward(d_E, d_enc, d_dW, d_grad, dE)
    torch.cuda.synchronize()

    dW64 = oracle.bf16_bits_to_f64(dW)
    want = None
    for b in range(B):
        r = oracle.hyper_encode_backward(E, "bf16", ref[b][1], enc, dW64[b])
        if want is None:
            want = r
        else:
            want["dE"] += r["dE"]
            if want["pos"] is not None:
                want["pos"] += r["pos"]
            for gl, rl in zip(want["layers"], r["layers"]):
                for k in gl:
                    gl[k] += rl[k]
    worst = {}
    _check("dE", dE.cpu().numpy(), want["dE"], worst)
    if enc["pos"] is not None:
        _check("pos", oracle.bf16_bits_to_f64(storage_to_host(d_grad.params["pos"], "bf16")), want["pos"], worst)
    for l, gl in enumerate(want["layers"]):
        for k, w in gl.items():
            t = d_grad.params["layers"][l][k]
            got = oracle.bf16_bits_to_f64(storage_to_host(t, "bf16")) if k.startswith("w_") else t.cpu().numpy()
            _check(f"layer {l} {k}", got, w, worst)
    ctx.close()
    top = sorted(worst.items(), key=lambda kv: -kv[1][0])[:3]
    print("  worst tensors (max, mean): " + ", ".join(f"{k} {a:.4f} {m:.5f}" for k, (a, m) in top), flush=True)
    return worst


@pytest.mark.parametrize("B,N,V,d,M,cap,n_layers,n_heads,d_ff,attn_only,with_pos", [
    (3, 300, 1000, 256, 3, 200, 2, 4, 512, False, True),       # two transformer layers, the paper's M
    (2, 200, 500, 128, 5, 90, 1, 2, 0, True, True),            # one attention layer, deeper merges
    (2, 260, 700, 512, 3, 130, 1, 1, 192, False, False),       # one head of 512 features, no slot positions
    (5, 150, 400, 64, 4, 64, 3, 8, 64, False, True),           # heads of 8 features; weight gradients of 64 rows
    (1, 900, 3000, 1024, 3, 600, 1, 8, 1024, False, True),     # rows spanning several 256-row tiles
    (2, 150, 400, 256, 3, 20, 2, 4, 512, True, True),          # two attention layers on ~100 rows
])
def test_hyper_encode_backward_matches_oracle(B, N, V, d, M, cap, n_layers, n_heads, d_ff, attn_only, with_pos):
    print(f"[case] hyper_encode_backward B={B} d={d} M={M} cap={cap} layers={n_layers} heads={n_heads} "
          f"d_ff={d_ff} attention_only={attn_only}", flush=True)
    _run_case(B, N, V, d, M, cap, n_layers, n_heads, d_ff, attn_only, with_pos, seed=13 * B + d)


def test_backward_over_more_rows_than_one_pass():
    """40 x 600 x 3 = 72000 slot rows: two passes; the matrix gradients of the second add to the first's."""
    print("[case] hyper_encode_backward two passes", flush=True)
    _run_case(40, 1500, 3000, 64, 3, 600, 1, 2, 64, False, True, seed=79, lens_zero=False)


def test_backward_accumulates_into_dE_and_overwrites_the_rest():
    import torch
    from paper_2506_01084_amd import api

    B, N, V, d, M, cap = 2, 200, 300, 128, 3, 80
    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=5)
    tokens = wl.make_tokens(cfg)
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype="bf16")
    gpu_encode(ctx, tokens, None)
    d_E = torch_storage(wl.make_embeddings(cfg), "bf16")
    enc = wl.make_encoder(cfg, n_layers=1, n_heads=2, d_ff=128)
    d_enc = encoder_to_device(enc, "bf16")
    d_dW = torch_storage(wl.normal_matrix(9, B * cap, d, 1.0, "bf16").reshape(B, cap, d), "bf16")
    g1, g2 = _grad_buffers(enc), _grad_buffers(enc)
    dE = torch.zeros((V, d), dtype=torch.float32, device="cuda")
    ctx.hyper_encode_backward(d_E, d_enc, d_dW, g1, dE)
    once = dE.clone()
    ctx.hyper_encode_backward(d_E, d_enc, d_dW, g2, dE)
    torch.cuda.synchronize()
    assert torch.allclose(dE, 2 * once, rtol=1e-3, atol=1e-5)          # float atomics: order may differ
    for k in g1.params["layers"][0]:
        a, b = g1.params["layers"][0][k], g2.params["layers"][0][k]
        if k.startswith("w_"):
            assert torch.equal(a, b), k                                  # same kernels, same order: same bits
        else:
            assert torch.allclose(a, b, rtol=1e-3, atol=1e-4), k         # (float atomics)
    # argument errors
    lib, h = ctx._lib, ctx._h
    import ctypes
    assert lib.z2z_hyper_encode_backward(h, None, ctypes.byref(d_enc.desc), d_dW.data_ptr(),
                                         ctypes.byref(g1.desc), dE.data_ptr(), 0, None) == -1
    assert lib.z2z_hyper_encode_backward(h, d_E.data_ptr(), ctypes.byref(d_enc.desc), d_dW.data_ptr(),
                                         ctypes.byref(g1.desc), None, 0, None) == -1
    assert lib.z2z_hyper_encode_backward(h, d_E.data_ptr(), ctypes.byref(d_enc.desc), d_dW.data_ptr(),
                                         ctypes.byref(g1.desc), dE.data_ptr(), 2, None) == -1        # unknown flag
    # the kept-rows flag without a preceding hyper_encode_keep
    assert lib.z2z_hyper_encode_backward(h, d_E.data_ptr(), ctypes.byref(d_enc.desc), d_dW.data_ptr(),
                                         ctypes.byref(g1.desc), dE.data_ptr(), api.ENC_KEPT, None) == -1
    two = _grad_buffers(wl.make_encoder(cfg, n_layers=2, n_heads=2, d_ff=128))
    assert lib.z2z_hyper_encode_backward(h, d_E.data_ptr(), ctypes.byref(d_enc.desc), d_dW.data_ptr(),
                                         ctypes.byref(two.desc), dE.data_ptr(), 0, None) == -1
    ctx.close()


def test_backward_on_the_rows_a_keeping_forward_left():
    """hyper_encode_keep writes the same W_hyper as hyper_encode (to the oracle's tolerance; the feed-forward
    pre-activation is rounded once more) and leaves the rows; backward with the flag gives what backward without
    it gives (the same kernels on the same rows: equal bits for the matrices), and consumes the rows."""
    import ctypes
    import torch
    from paper_2506_01084_amd import api

    B, N, V, d, M, cap = 3, 300, 1000, 256, 3, 200
    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=41)
    print("[case] hyper_encode_keep + backward on kept rows", flush=True)
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    lens = np.full(B, N, dtype=np.int32)
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype="bf16")
    gpu_encode(ctx, tokens, lens)
    ref = oracle_encode_batch(tokens, lens, V, M, cap)
    d_E = torch_storage(E, "bf16")
    enc = wl.make_encoder(cfg, n_layers=2, n_heads=4, d_ff=512)
    d_enc = encoder_to_device(enc, "bf16")
    d_dW = torch_storage(wl.normal_matrix(9, B * cap, d, 1.0, "bf16").reshape(B, cap, d), "bf16")
    g_plain, g_kept = _grad_buffers(enc), _grad_buffers(enc)
    dE_plain = torch.zeros((V, d), dtype=torch.float32, device="cuda")
    dE_kept = torch.zeros((V, d), dtype=torch.float32, device="cuda")
    ctx.hyper_encode_backward(d_E, d_enc, d_dW, g_plain, dE_plain)
    d_W = torch.full((B, cap, d), 5.0, dtype=torch.bfloat16, device="cuda")
    ctx.hyper_encode_keep(d_E, d_enc, d_W)
    ctx.hyper_encode_backward(d_E, d_enc, d_dW, g_kept, dE_kept, kept=True)
    torch.cuda.synchronize()
    W = storage_to_host(d_W, "bf16")
    for b in range(B):
        entries = ref[b][1]
        want = oracle.hyper_encode(E, "bf16", entries, cap, enc, rounded=False)
        got = oracle.bf16_bits_to_f64(W[b])
        scale = np.maximum(1.0, np.abs(want).max(axis=-1, keepdims=True))
        assert (np.abs(got - want) / scale).max() <= 2e-2                  # the forward test's bar
        assert (W[b, len(entries):] == 0).all()
    assert torch.allclose(dE_kept, dE_plain, rtol=1e-3, atol=1e-5)
    assert torch.equal(g_kept.params["pos"], g_plain.params["pos"]) or torch.allclose(
        g_kept.params["pos"].float(), g_plain.params["pos"].float(), rtol=2e-2, atol=1e-3)     # (float atomics)
    for l in range(2):
        for k in g_plain.params["layers"][l]:
            a, b_ = g_kept.params["layers"][l][k], g_plain.params["layers"][l][k]
            if k.startswith("w_"):
                assert torch.equal(a, b_), (l, k)
            else:
                assert torch.allclose(a, b_, rtol=1e-3, atol=1e-4), (l, k)
    # the rows are consumed: a second backward with the flag is refused; so is one after another encoder shape
    lib, h = ctx._lib, ctx._h
    args = (h, d_E.data_ptr(), ctypes.byref(d_enc.desc), d_dW.data_ptr(), ctypes.byref(g_kept.desc),
            dE_kept.data_ptr(), api.ENC_KEPT, None)
    assert lib.z2z_hyper_encode_backward(*args) == -1
    ctx.hyper_encode_keep(d_E, d_enc, d_W)
    one = wl.make_encoder(cfg, n_layers=1, n_heads=4, d_ff=512)
    d_one, g_one = encoder_to_device(one, "bf16"), _grad_buffers(one)
    assert lib.z2z_hyper_encode_backward(h, d_E.data_ptr(), ctypes.byref(d_one.desc), d_dW.data_ptr(),
                                         ctypes.byref(g_one.desc), dE_kept.data_ptr(), api.ENC_KEPT, None) == -1
    # a codebook change between the keeping call and the backward call makes the kept rows stale: refused
    ctx.hyper_encode_keep(d_E, d_enc, d_W)
    d_one_code = torch.zeros((cfg["B"], 1), dtype=torch.int32, device="cuda")
    scratch_n = torch.empty(cfg["B"], dtype=torch.int32, device="cuda")
    scratch_st = torch.empty(cfg["B"], dtype=torch.int32, device="cuda")
    ctx.lzw_decode(d_one_code, None, None, scratch_n, scratch_st, api.APPEND)
    assert lib.z2z_hyper_encode_backward(*args) == -1
    ctx.close()
    # more slot rows than one pass holds: keeping is refused (the plain backward takes passes)
    ctx = api.Context(B=40, V=V, M=3, cap=600, d=64, dtype="bf16")
    small = wl.make_encoder(dict(cfg, d=64), n_layers=1, n_heads=2, d_ff=64)
    d_small = encoder_to_device(small, "bf16")
    E64 = torch.zeros((V, 64), dtype=torch.bfloat16, device="cuda")
    W64 = torch.zeros((40, 600, 64), dtype=torch.bfloat16, device="cuda")
    assert ctx._lib.z2z_hyper_encode_keep(ctx._h, E64.data_ptr(), ctypes.byref(d_small.desc), W64.data_ptr(),
                                          None) == -4        # Z2Z_EUNSUPPORTED
    ctx.close()


def test_full_size_c2_two_layer_transformer_sampled_entries():
    """Configuration 2's codebooks through the backward pass of the encoder the benchmark times (two transformer
    layers, 32 heads, d_ff = 4 d), in the launch shapes of the full call: dW_hyper is zero except at a few
    sampled entries, so the gradients are sums over those entries alone, which the oracle computes one by
    one."""
    import time
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.CONFIGS["c2"]
    B, V, M, cap, d = cfg["B"], cfg["V"], cfg["M"], cfg["cap"], cfg["d"]
    t0 = time.time()
    print("[case] full size hyper_encode_backward c2", flush=True)
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype="bf16")
    gpu_encode(ctx, tokens, None)
    ref = oracle_encode_batch(tokens, np.full(B, cfg["N"], dtype=np.int32), V, M, cap)
    d_E = torch_storage(E, "bf16")
    enc = wl.make_encoder(cfg, n_layers=2, n_heads=32)
    d_enc = encoder_to_device(enc, "bf16")
    d_grad = _grad_buffers(enc)
    picks = []
    for b in (0, 3, 7):
        C = len(ref[b][1])
        picks += [(b, i) for i in (0, C // 3, C - 1)]
    dW = np.zeros((B, cap, d), dtype=np.uint16)
    rows = wl.normal_matrix(31, len(picks), d, 1.0, "bf16")
    for k, (b, i) in enumerate(picks):
        dW[b, i] = rows[k]
    d_dW = torch_storage(dW, "bf16")
    dE = torch.zeros((V, d), dtype=torch.float32, device="cuda")
    ctx.hyper_encode_backward(d_E, d_enc, d_dW, d_grad, dE)
    torch.cuda.synchronize()
    print(f"  GPU pass done {time.time() - t0:.1f}s", flush=True)
    want = oracle.hyper_encode_backward(E, "bf16", [ref[b][1][i] for b, i in picks], enc,
                                        oracle.bf16_bits_to_f64(rows))
    print(f"  oracle done {time.time() - t0:.1f}s", flush=True)
    worst = {}
    touched = sorted({t for b, i in picks for t in ref[b][1][i]})
    got_dE = dE.cpu().numpy()
    _check("dE rows of the entries' tokens", got_dE[touched], want["dE"][touched], worst)
    untouched = np.ones(V, dtype=bool)
    untouched[touched] = False
    assert (got_dE[untouched] == 0).all()
    _check("pos", oracle.bf16_bits_to_f64(storage_to_host(d_grad.params["pos"], "bf16")), want["pos"], worst)
    for l, gl in enumerate(want["layers"]):
        for k, w in gl.items():
            t = d_grad.params["layers"][l][k]
            got = oracle.bf16_bits_to_f64(storage_to_host(t, "bf16")) if k.startswith("w_") else t.cpu().numpy()
            _check(f"layer {l} {k}", got, w, worst)
    top = sorted(worst.items(), key=lambda kv: -kv[1][0])[:4]
    print("  worst tensors (max, mean): " + ", ".join(f"{k} {a:.4f} {m:.5f}" for k, (a, m) in top), flush=True)
    print(f"  compared {time.time() - t0:.1f}s", flush=True)
    ctx.close()
