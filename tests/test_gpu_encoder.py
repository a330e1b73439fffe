"""GPU parity: hyper_encode (the learned hyper-encoder of section 2.2: attention / transformer layers over an
entry's padded slots, mean of the real slots) through the C ABI against the float64 oracle.

Bar.  The HIP path keeps the residual stream (slot inputs, the sums after the attention and the feed-forward
block) in fp32 from the gather to the final mean; what feeds a matrix product is bf16 (LayerNorm outputs, q|k|v,
attention output, the GELU output) and accumulation is fp32.  The oracle computes in float64 from the same
stored parameters and rounds once.  Each rounding is a relative 2^-9 of the rounded value and reaches the
output only through a weight matrix (none sits on the stream itself, where it would arrive with weight 1); with
random-init parameters of the scale used here every product maps order-1 activations to order-1 activations,
so the 5 L roundings of an L-layer encoder and the one of the result add in quadrature: sqrt(11) * 2^-9 =
6.5e-3 for two layers as the typical error of an element, about twice that for the worst element of a tensor.
The tolerance is 2e-2 * max(1, largest |h| of the row) per element, and a row's mean error has to stay below a
quarter of that (the largest seen over 2277 random shapes and modes was 1.29e-2; with the stream rounded to
bf16 after every block it had been 2.24e-2).
"""
import numpy as np
import pytest

import oracle
from paper_2506_01084_amd import workloads as wl

from helpers import encoder_to_device, gpu_encode, oracle_encode_batch, storage_to_host, torch_storage

pytestmark = pytest.mark.gpu

TOL = 2e-2


def _compare(got_bits, ref64, label):
    got = oracle.bf16_bits_to_f64(got_bits)
    scale = np.maximum(1.0, np.abs(ref64).max(axis=-1, keepdims=True))
    err = np.abs(got - ref64) / scale
    assert err.max() <= TOL, f"{label}: max error {err.max():.4f}"
    assert err.mean(axis=-1).max() <= TOL / 4, f"{label}: mean row error {err.mean(axis=-1).max():.4f}"
    return float(err.max()), float(err.mean())


def _setup(cfg, lens):
    import torch
    from paper_2506_01084_amd import api

    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    ctx = api.Context(B=cfg["B"], V=cfg["V"], M=cfg["M"], cap=cfg["cap"], d=cfg["d"], dtype="bf16")
    gpu_encode(ctx, tokens, lens)
    ref = oracle_encode_batch(tokens, lens, cfg["V"], cfg["M"], cfg["cap"])
    d_E = torch_storage(E, "bf16")
    torch.cuda.synchronize()
    return ctx, ref, E, d_E


@pytest.mark.parametrize("B,N,V,d,M,cap,n_layers,n_heads,d_ff,attn_only,with_pos", [
    (3, 300, 1000, 256, 3, 200, 2, 4, 512, False, True),       # two transformer layers, the paper's M
    (2, 200, 500, 128, 5, 90, 1, 2, 0, True, True),            # one attention layer, deeper merges
    (2, 260, 700, 512, 3, 130, 1, 1, 192, False, False),       # one head as wide as a wave's 512 features
    (5, 150, 400, 64, 4, 64, 3, 8, 64, False, True),           # heads of 8 features (one lane each)
    (1, 900, 3000, 1024, 3, 600, 1, 8, 1024, False, True),     # rows spanning several 256-row tiles
    (2, 150, 400, 256, 3, 64, 2, 4, 512, False, True),         # 384 slot rows: the few-rows kernel for the layers
    (1, 100, 300, 384, 4, 20, 1, 6, 1152, False, True),        # 80 rows, K = 384 and 1152 (3 and 9 slices of 128)
    (2, 300, 600, 1024, 3, 40, 2, 8, 2048, False, True),       # 240 rows, K = 1024 and 2048: the tile kernel with K split
    (4, 400, 800, 512, 3, 70, 1, 4, 1024, False, True),        # 840 slot rows at most, few tiles: K split beyond 512 rows
])
def test_hyper_encode_matches_oracle_every_entry(B, N, V, d, M, cap, n_layers, n_heads, d_ff, attn_only, with_pos):
    import torch

    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=11 * B + d)
    print(f"[case] hyper_encode B={B} d={d} M={M} cap={cap} layers={n_layers} heads={n_heads} d_ff={d_ff} "
          f"attention_only={attn_only}", flush=True)
    lens = wl.make_lens(cfg, ragged=True)
    if B > 1:
        lens[1] = 0
    ctx, ref, E, d_E = _setup(cfg, lens)
    enc = wl.make_encoder(cfg, n_layers=n_layers, n_heads=n_heads, d_ff=d_ff, attention_only=attn_only,
                          with_pos=with_pos)
    d_enc = encoder_to_device(enc, "bf16")
    d_W = torch.full((B, cap, d), 7.0, dtype=torch.bfloat16, device="cuda")
    ctx.hyper_encode(d_E, d_enc, d_W)
    torch.cuda.synchronize()
    W = storage_to_host(d_W, "bf16")
    worst = 0.0
    for b in range(B):
        entries = ref[b][1]
        want = oracle.hyper_encode(E, "bf16", entries, cap, enc, rounded=False)
        if entries:
            worst = max(worst, _compare(W[b, :len(entries)], want[:len(entries)], f"seq {b}")[0])
        assert (W[b, len(entries):] == 0).all(), f"seq {b}: rows of missing entries must be zero"
    print(f"  worst relative error {worst:.4f}", flush=True)
    ctx.close()


def test_incremental_modes_recompute_the_same_rows():
    """A row's result depends on that entry alone, so recomputing a range of entries (from d_first, or the last
    n) reproduces the rows of the full pass and leaves every other row untouched.  With the same kernels the
    bits are the same; a pass of few rows takes its dense layers on another kernel (another summation order),
    and then the rows agree to the rounding of the bf16 activations."""
    import torch

    B, N, V, d, M, cap = 4, 400, 800, 256, 3, 256
    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=5)
    lens = wl.make_lens(cfg, ragged=True)
    ctx, ref, E, d_E = _setup(cfg, lens)
    enc = wl.make_encoder(cfg, n_layers=2, n_heads=4, d_ff=256)
    d_enc = encoder_to_device(enc, "bf16")
    full = torch.zeros((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.hyper_encode(d_E, d_enc, full)
    sizes = np.array([len(r[1]) for r in ref])
    # from d_first
    first = np.maximum(sizes - np.array([3, 50, 0, 7]), 0).astype(np.int32)
    part = torch.full((B, cap, d), -3.0, dtype=torch.bfloat16, device="cuda")
    ctx.hyper_encode(d_E, d_enc, part, torch.from_numpy(first).cuda(), 50)
    # the last 2
    last = torch.full((B, cap, d), -3.0, dtype=torch.bfloat16, device="cuda")
    ctx.hyper_encode(d_E, d_enc, last, None, 2)
    torch.cuda.synchronize()
    f, p, l = (storage_to_host(t, "bf16") for t in (full, part, last))
    untouched = oracle.f64_to_bf16_bits(np.array([-3.0]))[0]
    for b in range(B):
        C = sizes[b]
        assert np.array_equal(p[b, first[b]:C], f[b, first[b]:C])
        assert (p[b, :first[b]] == untouched).all() and (p[b, C:] == untouched).all()
        lo = max(C - 2, 0)
        if C > lo:
            _compare(l[b, lo:C], oracle.bf16_bits_to_f64(f[b, lo:C]), f"last two of seq {b}")
        assert (l[b, :lo] == untouched).all() and (l[b, C:] == untouched).all()
    ctx.close()


def test_unsupported_shapes_are_refused():
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c2"], B=1, N=64, V=100, d=192, M=3, cap=16)
    ctx = api.Context(B=1, V=100, M=3, cap=16, d=192, dtype="bf16")
    ctx.reset()
    E = torch.zeros((100, 192), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((1, 16, 192), dtype=torch.bfloat16, device="cuda")
    enc = encoder_to_device(wl.make_encoder(cfg, n_layers=1, n_heads=4, d_ff=64), "bf16")     # heads of 48 features
    with pytest.raises(api.Z2ZError):
        ctx.hyper_encode(E, enc, W)
    ctx.close()


def test_full_size_c2_two_layer_transformer_sampled_entries():
    """Configuration 2's codebooks through the encoder the benchmark times (two transformer layers, 32 heads,
    d_ff = 4 d): sampled entries against the oracle, for the full pass (tile kernel) and for the newest entry of
    every sequence recomputed alone (the few-rows kernel, K up to 16384)."""
    import time
    import torch

    cfg = wl.CONFIGS["c2"]
    B, cap, d = cfg["B"], cfg["cap"], cfg["d"]
    t0 = time.time()
    print("[case] full size hyper_encode c2", flush=True)
    ctx, ref, E, d_E = _setup(cfg, np.full(B, cfg["N"], dtype=np.int32))
    enc = wl.make_encoder(cfg, n_layers=2, n_heads=32)
    d_enc = encoder_to_device(enc, "bf16")
    d_W = torch.zeros((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.hyper_encode(d_E, d_enc, d_W)
    torch.cuda.synchronize()
    full = storage_to_host(d_W, "bf16")
    d_W2 = torch.zeros((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.hyper_encode(d_E, d_enc, d_W2, None, 1)
    torch.cuda.synchronize()
    newest = storage_to_host(d_W2, "bf16")
    print(f"  GPU passes done {time.time() - t0:.1f}s", flush=True)
    picks = []
    for b in (0, 3, 7):
        C = len(ref[b][1])
        picks += [(b, i) for i in (0, 1, C // 3, C - 1)]
    want = oracle.hyper_encode(E, "bf16", [ref[b][1][i] for b, i in picks], len(picks), enc, rounded=False)
    print(f"  oracle done {time.time() - t0:.1f}s", flush=True)
    for k, (b, i) in enumerate(picks):
        e_full = _compare(full[b, i:i + 1], want[k:k + 1], f"full pass, seq {b} entry {i}")
        if i == len(ref[b][1]) - 1:
            e_new = _compare(newest[b, i:i + 1], want[k:k + 1], f"newest entry, seq {b}")
            print(f"  seq {b} entry {i} (len {len(ref[b][1][i])}): full {e_full[0]:.4f}, alone {e_new[0]:.4f}", flush=True)
    for b in range(B):
        C = len(ref[b][1])
        assert (newest[b, :C - 1] == 0).all() and (newest[b, C:] == 0).all()
    ctx.close()


def test_codebooks_larger_than_one_pass_and_edge_shapes():
    """More slot rows than the work space of one pass holds (65536): the entries go in several passes over
    entry ranges.  Also M = 8 (the largest), an empty batch of codebooks, and cap = 0."""
    import torch
    from paper_2506_01084_amd import api

    # 40 x 600 x 3 = 72000 slot rows -> two passes of 546 and 54 entries per sequence
    B, N, V, d, M, cap = 40, 1500, 3000, 128, 3, 600
    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.2, seed=77)
    lens = wl.make_lens(cfg, ragged=True)
    ctx, ref, E, d_E = _setup(cfg, lens)
    enc = wl.make_encoder(cfg, n_layers=1, n_heads=2, d_ff=128)
    d_enc = encoder_to_device(enc, "bf16")
    d_W = torch.full((B, cap, d), 3.0, dtype=torch.bfloat16, device="cuda")
    ctx.hyper_encode(d_E, d_enc, d_W)
    torch.cuda.synchronize()
    W = storage_to_host(d_W, "bf16")
    assert max(len(r[1]) for r in ref) > 546, "the case must reach the second pass"
    for b in (0, 7, 39):
        entries = ref[b][1]
        want = oracle.hyper_encode(E, "bf16", entries, cap, enc, rounded=False)
        _compare(W[b, :len(entries)], want[:len(entries)], f"two passes, seq {b}")
        assert (W[b, len(entries):] == 0).all()
    ctx.close()

    # M = 8
    B, N, V, d, M, cap = 2, 600, 40, 64, 8, 120
    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.0, seed=78)
    tokens = np.empty((B, N), dtype=np.int32)           # repetitive streams: entries grow to the full M slots
    tokens[0] = 5
    tokens[1] = np.tile(np.array([1, 2, 3], dtype=np.int32), N // 3)
    E = wl.make_embeddings(cfg)
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype="bf16")
    gpu_encode(ctx, tokens, None)
    ref = oracle_encode_batch(tokens, np.full(B, N, dtype=np.int32), V, M, cap)
    d_E = torch_storage(E, "bf16")
    assert max(len(e) for e in ref[0][1]) == 8
    enc = wl.make_encoder(cfg, n_layers=1, n_heads=4, d_ff=64)
    d_W = torch.zeros((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.hyper_encode(d_E, encoder_to_device(enc, "bf16"), d_W)
    torch.cuda.synchronize()
    W = storage_to_host(d_W, "bf16")
    for b in range(B):
        want = oracle.hyper_encode(E, "bf16", ref[b][1], cap, enc, rounded=False)
        _compare(W[b, :len(ref[b][1])], want[:len(ref[b][1])], f"M = 8, seq {b}")
    # no entries at all (fresh codebooks): every row zero, nothing faults
    ctx.reset()
    d_W.fill_(5.0)
    ctx.hyper_encode(d_E, encoder_to_device(enc, "bf16"), d_W)
    ctx.hyper_encode(d_E, encoder_to_device(enc, "bf16"), d_W, None, 1)
    torch.cuda.synchronize()
    assert (storage_to_host(d_W, "bf16") == 0).all()
    ctx.close()

    # cap = 0: nothing to do
    ctx = api.Context(B=2, V=40, M=3, cap=0, d=64, dtype="bf16")
    ctx.reset()
    cfg0 = wl.scaled(cfg, M=3)
    ctx.hyper_encode(d_E, encoder_to_device(wl.make_encoder(cfg0, n_layers=1, n_heads=4, d_ff=64), "bf16"),
                     torch.zeros((2, 0, 64), dtype=torch.bfloat16, device="cuda"))
    torch.cuda.synchronize()
    ctx.close()


def test_hyper_encode_replays_in_a_graph():
    """After one eager call (which allocates the work space) the call enqueues kernels only, with the row count
    read on the device: a captured graph replays it on codebooks that grew in between."""
    import torch
    from paper_2506_01084_amd import api

    B, N, V, d, M, cap = 4, 300, 500, 256, 3, 400
    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=21)
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    d_E = torch_storage(E, "bf16")
    enc = wl.make_encoder(cfg, n_layers=2, n_heads=4, d_ff=256)
    d_enc = encoder_to_device(enc, "bf16")
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype="bf16")
    half = np.full(B, N // 2, dtype=np.int32)
    gpu_encode(ctx, tokens[:, :N // 2].copy(), half)
    d_W = torch.zeros((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.hyper_encode(d_E, d_enc, d_W)                    # eager: sizes the work space
    torch.cuda.synchronize()
    eager_half = storage_to_host(d_W, "bf16").copy()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            ctx.hyper_encode(d_E, d_enc, d_W)
    torch.cuda.current_stream().wait_stream(side)
    d_W.zero_()
    g.replay()
    torch.cuda.synchronize()
    assert np.array_equal(storage_to_host(d_W, "bf16"), eager_half)
    # the codebooks grow (second half of the tokens appended), the same graph is replayed
    gpu_encode(ctx, tokens[:, N // 2:].copy(), half, flags=api.APPEND)
    ref = []
    for b in range(B):                                  # the oracle's chunked encoder: same two chunks
        st = oracle.LZWStream(V, M, cap)
        st.encode_chunk(tokens[b, :N // 2].tolist())
        st.encode_chunk(tokens[b, N // 2:].tolist())
        ref.append((None, list(st.entries)))
    for rep in range(2):
        d_W.zero_()
        g.replay()
        torch.cuda.synchronize()
        W = storage_to_host(d_W, "bf16")
        for b in range(B):
            entries = ref[b][1]
            want = oracle.hyper_encode(E, "bf16", entries, cap, enc, rounded=False)
            _compare(W[b, :len(entries)], want[:len(entries)], f"replay {rep}, seq {b}")
            assert (W[b, len(entries):] == 0).all()
    ctx.close()


def test_argument_errors_of_the_newer_entry_points():
    """Bad arguments are refused on the host, before anything is enqueued."""
    import ctypes
    import torch
    from paper_2506_01084_amd import api

    lib = api.load_library()
    ctx = api.Context(B=1, V=100, M=3, cap=8, d=64, dtype="bf16")
    ctx.reset()
    E = torch.zeros((100, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((1, 8, 64), dtype=torch.bfloat16, device="cuda")
    cfg = wl.scaled(wl.CONFIGS["c2"], B=1, N=8, V=100, d=64, M=3, cap=8)
    enc = encoder_to_device(wl.make_encoder(cfg, n_layers=1, n_heads=2, d_ff=64), "bf16")
    EINVAL = -1
    h = ctx._h
    # no encoder, no layers, too many layers, a missing matrix
    assert lib.z2z_hyper_encode(h, E.data_ptr(), None, W.data_ptr(), None, 0, None) == EINVAL
    desc = api.EncoderDesc.from_buffer_copy(enc.desc)
    desc.n_layers = 9
    assert lib.z2z_hyper_encode(h, E.data_ptr(), ctypes.byref(desc), W.data_ptr(), None, 0, None) == EINVAL
    arr = (api.EncoderLayer * 1)()
    ctypes.memmove(arr, enc._arr, ctypes.sizeof(arr))
    arr[0].w_o = None
    desc = api.EncoderDesc.from_buffer_copy(enc.desc)
    desc.layers = ctypes.cast(arr, ctypes.POINTER(api.EncoderLayer))
    assert lib.z2z_hyper_encode(h, E.data_ptr(), ctypes.byref(desc), W.data_ptr(), None, 0, None) == EINVAL
    # backward: rows must be B * rows_per_seq; the lse of the forward pass is required
    z = torch.zeros(8, dtype=torch.float32, device="cuda")
    t = torch.zeros(8, dtype=torch.int32, device="cuda")
    Hh = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    assert lib.z2z_extended_nll_backward(h, Hh.data_ptr(), 8, 3, E.data_ptr(), W.data_ptr(), t.data_ptr(), z.data_ptr(),
                                         None, Hh.data_ptr(), E.data_ptr(), W.data_ptr(), None) == EINVAL
    assert lib.z2z_extended_nll_backward(h, Hh.data_ptr(), 8, 8, E.data_ptr(), W.data_ptr(), t.data_ptr(), None, None,
                                         Hh.data_ptr(), E.data_ptr(), W.data_ptr(), None) == EINVAL
    # prefill: flags must be RESET or APPEND, outputs required
    i32 = torch.zeros(8, dtype=torch.int32, device="cuda")
    assert lib.z2z_codebook_prefill(h, i32.data_ptr(), i32.data_ptr(), None, 1, 7, i32.data_ptr(), i32.data_ptr(), None) == EINVAL
    assert lib.z2z_codebook_prefill(h, i32.data_ptr(), i32.data_ptr(), None, 1, api.RESET, None, i32.data_ptr(), None) == EINVAL
    ctx.close()
