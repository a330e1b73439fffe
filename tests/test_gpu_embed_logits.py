"""GPU parity: hyper_embed and extended_logits through the C ABI against the float64 oracle.

Tolerances (the stated bars; the arithmetic behind them is in the design notes):
  hyper_embed   |gpu - ref| <= tol * sum_j a_j |E[t_j]| per element, tol = 1e-5 (f32) / 2e-2 (bf16)
  logits        max_v |gpu - ref| / max_v |ref| <= 2e-2 per row; max and lse within 2e-2 * max(1, |ref|)
  argmax        identical wherever the oracle's top-2 gap exceeds 1e-2
"""
import time

import numpy as np
import pytest

import oracle
from paper_2506_01084_amd import workloads as wl

from helpers import (check_logits_rows, gpu_encode, hyper_embed_bound, oracle_encode_batch, storage_to_host,
                     torch_storage)

pytestmark = pytest.mark.gpu


def _make_ctx(cfg):
    from paper_2506_01084_amd import api

    w = wl.make_pool_weights(cfg)
    return api.Context(B=cfg["B"], V=cfg["V"], M=cfg["M"], cap=cfg["cap"], d=cfg["d"], dtype=cfg["dtype"],
                       pool=cfg["pool"], w=w.tolist()), w


def _encode(ctx, cfg, tokens, lens=None):
    lens = wl.make_lens(cfg) if lens is None else lens
    gpu_encode(ctx, tokens, lens)
    return oracle_encode_batch(tokens, lens, cfg["V"], cfg["M"], cfg["cap"])


def _embed_gpu(ctx, cfg, E_host):
    import torch

    d_E = torch_storage(E_host, cfg["dtype"])
    poison = 1.0 if cfg["dtype"] == "f32" else 1.0
    d_W = torch.full((cfg["B"], cfg["cap"], cfg["d"]), poison, dtype=ctx.torch_dtype, device="cuda")
    ctx.hyper_embed(d_E, d_W)
    torch.cuda.synchronize()
    return d_E, d_W


def _check_embed(cfg, ref, E_host, d_W, w, seqs=None):
    tol = 1e-5 if cfg["dtype"] == "f32" else 2e-2
    W_host = storage_to_host(d_W, cfg["dtype"])
    worst = 0.0
    refW = {}
    for b in (range(cfg["B"]) if seqs is None else seqs):
        entries = ref[b][1]
        Wr = oracle.hyper_embed(E_host, cfg["dtype"], entries, cfg["cap"], cfg["pool"], w)
        refW[b] = Wr
        got = oracle.to_f64(W_host[b], cfg["dtype"])
        want = oracle.to_f64(Wr, cfg["dtype"])
        C = len(entries)
        assert (got[C:] == 0).all(), f"seq {b}: rows beyond the codebook must be zero"
        bound = hyper_embed_bound(E_host, cfg["dtype"], entries, cfg["pool"], w, cfg["cap"])
        err = np.abs(got - want)
        assert (err <= tol * bound + 1e-30).all(), f"seq {b}: hyper_embed error {np.max(err / (bound + 1e-30))}"
        worst = max(worst, float(np.max(err[:C] / (bound[:C] + 1e-30))) if C else 0.0)
    return refW, worst


# ---------------------------------------------------------------------------------------------------
# config 1 at full size: everything, element by element, including the full logits matrix
# ---------------------------------------------------------------------------------------------------
def test_c1_full_path_elementwise():
    import torch

    cfg = wl.CONFIGS["c1"]
    print("[case] c1 full path", flush=True)
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    rows_per_seq = cfg["N"]
    rows = cfg["B"] * rows_per_seq
    H = wl.make_hidden(cfg, rows)
    ctx, w = _make_ctx(cfg)
    ref = _encode(ctx, cfg, tokens)
    d_E, d_W = _embed_gpu(ctx, cfg, E)
    refW, worst = _check_embed(cfg, ref, E, d_W, w)
    print(f"  hyper_embed worst relative-to-scale error {worst:.3e}", flush=True)

    d_H = torch_storage(H, cfg["dtype"])
    am = torch.empty(rows, dtype=torch.int32, device="cuda")
    mx = torch.empty(rows, dtype=torch.float32, device="cuda")
    lse = torch.empty(rows, dtype=torch.float32, device="cuda")
    full = torch.full((rows, cfg["V"] + cfg["cap"]), 123.0, dtype=torch.float32, device="cuda")
    ctx.extended_logits(d_H, rows_per_seq, d_E, d_W, am, mx, lse, full)
    torch.cuda.synchronize()
    am_h, mx_h, lse_h, full_h = am.cpu().numpy(), mx.cpu().numpy(), lse.cpu().numpy(), full.cpu().numpy()
    for b in range(cfg["B"]):
        sl = slice(b * rows_per_seq, (b + 1) * rows_per_seq)
        r = oracle.extended_logits(H[sl], E, refW[b], len(ref[b][1]), cfg["dtype"])
        errs = check_logits_rows(r, am_h[sl], mx_h[sl], lse_h[sl], full_h[sl], V=cfg["V"])
        print(f"  seq {b}: C={len(ref[b][1])} errors {errs}", flush=True)
    # without the full-logits output the reduced results are identical
    am2 = torch.empty_like(am); mx2 = torch.empty_like(mx); lse2 = torch.empty_like(lse)
    ctx.extended_logits(d_H, rows_per_seq, d_E, d_W, am2, mx2, lse2, None)
    torch.cuda.synchronize()
    assert torch.equal(am, am2) and torch.equal(mx, mx2) and torch.equal(lse, lse2)
    ctx.close()


# ---------------------------------------------------------------------------------------------------
# small shapes that span several tiles with ragged tails in every dimension
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,B,N,V,d,M,cap,pool", [
    ("bf16", 3, 200, 1000, 264, 3, 300, "mean"),       # nothing a multiple of the tile sizes
    ("bf16", 2, 130, 257, 72, 5, 140, "weighted"),
    ("f32", 2, 150, 300, 100, 4, 130, "weighted"),
    ("bf16", 4, 1, 700, 128, 3, 64, "mean"),           # one row per sequence (decode shape)
    ("bf16", 1, 384, 512, 512, 2, 0, "mean"),          # no hyper vocabulary at all
])
def test_small_ragged_shapes(dtype, B, N, V, d, M, cap, pool):
    import torch

    cfg = dict(name="small", B=B, N=max(N, 400), V=V, d=d, dtype=dtype, M=M, cap=cap, zipf_s=1.1, copy_frac=0.4,
               span=(2, 6), mode="motif", pool=pool, seed=77 + V)
    print(f"[case] small ragged {dtype} B={B} rows/seq={N} V={V} d={d} M={M} cap={cap} {pool}", flush=True)
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    rows = B * N
    H = wl.make_hidden(cfg, rows)
    ctx, w = _make_ctx(cfg)
    ref = _encode(ctx, cfg, tokens)
    d_E = torch_storage(E, dtype)
    if cap:
        _, d_W = _embed_gpu(ctx, cfg, E)
        refW, _ = _check_embed(cfg, ref, E, d_W, w)
    else:
        d_W = torch.empty((B, 0, d), dtype=ctx.torch_dtype, device="cuda")
        refW = {b: np.zeros((0, d), dtype=np.float32 if dtype == "f32" else np.uint16) for b in range(B)}
    d_H = torch_storage(H, dtype)
    am = torch.empty(rows, dtype=torch.int32, device="cuda")
    mx = torch.empty(rows, dtype=torch.float32, device="cuda")
    lse = torch.empty(rows, dtype=torch.float32, device="cuda")
    full = torch.full((rows, V + cap), 123.0, dtype=torch.float32, device="cuda")
    from paper_2506_01084_amd import api
    for strip in (0, 1, 3):
        ctx.set_option(api.OPT_LOGITS_STRIP, strip)
        ctx.extended_logits(d_H, N, d_E, d_W, am, mx, lse, full)
        torch.cuda.synchronize()
        am_h, mx_h, lse_h, full_h = am.cpu().numpy(), mx.cpu().numpy(), lse.cpu().numpy(), full.cpu().numpy()
        for b in range(B):
            sl = slice(b * N, (b + 1) * N)
            r = oracle.extended_logits(H[sl], E, refW[b], len(ref[b][1]), dtype)
            check_logits_rows(r, am_h[sl], mx_h[sl], lse_h[sl], full_h[sl], V=V)
    ctx.close()


def test_exact_ties_pick_lowest_index_and_masked_slots_never_win():
    """H = 0 makes every logit 0: argmax must be column 0 and lse = ln(V + C_b); then poison unused slots."""
    import math
    import torch

    cfg = dict(name="ties", B=2, N=120, V=333, d=64, dtype="bf16", M=3, cap=200, zipf_s=1.1, copy_frac=0.5,
               span=(2, 5), mode="motif", pool="mean", seed=5)
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    ctx, w = _make_ctx(cfg)
    ref = _encode(ctx, cfg, tokens)
    d_E, d_W = _embed_gpu(ctx, cfg, E)
    rows = cfg["B"] * 5
    d_H = torch.zeros((rows, cfg["d"]), dtype=torch.bfloat16, device="cuda")
    am = torch.empty(rows, dtype=torch.int32, device="cuda")
    mx = torch.empty(rows, dtype=torch.float32, device="cuda")
    lse = torch.empty(rows, dtype=torch.float32, device="cuda")
    ctx.extended_logits(d_H, 5, d_E, d_W, am, mx, lse, None)
    torch.cuda.synchronize()
    assert (am.cpu().numpy() == 0).all() and (mx.cpu().numpy() == 0).all()
    for b in range(cfg["B"]):
        C = len(ref[b][1])
        assert 0 < C < cfg["cap"]
        assert np.allclose(lse.cpu().numpy()[b * 5:(b + 1) * 5], math.log(cfg["V"] + C), atol=1e-4)
    # unused hyper slots hold huge rows: they must not change anything
    H = wl.make_hidden(cfg, rows)
    d_H = torch_storage(H, "bf16")
    ctx.extended_logits(d_H, 5, d_E, d_W, am, mx, lse, None)
    torch.cuda.synchronize()
    keep = (am.clone(), mx.clone(), lse.clone())
    d_Wp = d_W.clone()
    for b in range(cfg["B"]):
        d_Wp[b, len(ref[b][1]):] = 1000.0
    ctx.extended_logits(d_H, 5, d_E, d_Wp, am, mx, lse, None)
    torch.cuda.synchronize()
    assert torch.equal(am, keep[0]) and torch.equal(mx, keep[1]) and torch.equal(lse, keep[2])
    ctx.close()


def test_incremental_hyper_embed_only_touches_new_rows():
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c3"], B=4, N=1500, d=256, cap=2048)
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    ctx, w = _make_ctx(cfg)
    half = 700
    gpu_encode(ctx, np.ascontiguousarray(tokens[:, :half]), None)
    d_E, d_W = _embed_gpu(ctx, cfg, E)
    first = ctx.codebook()[2].clone()
    gpu_encode(ctx, np.ascontiguousarray(tokens[:, half:]), None, flags=api.APPEND)
    sentinel = d_W.clone()
    ctx.hyper_embed(d_E, d_W, first, max_new=8)          # a deliberately small launch hint
    torch.cuda.synchronize()
    # reference: embed everything from scratch
    d_W2 = torch.empty_like(d_W)
    ctx.hyper_embed(d_E, d_W2)
    torch.cuda.synchronize()
    size = ctx.codebook()[2].cpu().numpy()
    f = first.cpu().numpy()
    assert (size > f).all()
    for b in range(cfg["B"]):
        assert torch.equal(d_W[b, f[b]:size[b]], d_W2[b, f[b]:size[b]])
        assert torch.equal(d_W[b, :f[b]], sentinel[b, :f[b]])
        assert torch.equal(d_W[b, size[b]:], sentinel[b, size[b]:])
    # the snapshot-free form: only the last k entries of each sequence, k larger than some codebooks
    for k in (1, 5, 4000):
        d_W3 = torch.full_like(d_W, 3.0)
        ctx.hyper_embed(d_E, d_W3, None, max_new=k)
        torch.cuda.synchronize()
        for b in range(cfg["B"]):
            lo = max(int(size[b]) - k, 0)
            assert torch.equal(d_W3[b, lo:size[b]], d_W2[b, lo:size[b]])
            assert (d_W3[b, :lo] == 3.0).all() and (d_W3[b, size[b]:] == 3.0).all()
    ctx.close()


# ---------------------------------------------------------------------------------------------------
# full benchmark sizes, in the launch configuration the benchmark times: sampled rows vs the oracle
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,per_seq", [("c2", 6), ("c4", 8), ("c5", 3)])
def test_full_size_prefill_sampled_rows(name, per_seq):
    import torch

    cfg = wl.CONFIGS[name]
    t0 = time.time()
    print(f"[case] full size prefill {name}", flush=True)
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    rows_per_seq = cfg["N"]
    rows = cfg["B"] * rows_per_seq
    H = wl.make_hidden(cfg, rows)
    print(f"  inputs ready {time.time() - t0:.1f}s", flush=True)
    ctx, w = _make_ctx(cfg)
    ref = _encode(ctx, cfg, tokens)
    d_E, d_W = _embed_gpu(ctx, cfg, E)
    seqs = sorted(set([0, cfg["B"] - 1]))
    refW, worst = _check_embed(cfg, ref, E, d_W, w, seqs=seqs)
    print(f"  hyper_embed checked on sequences {seqs}: worst {worst:.3e}  {time.time() - t0:.1f}s", flush=True)
    d_H = torch_storage(H, cfg["dtype"])
    am = torch.empty(rows, dtype=torch.int32, device="cuda")
    mx = torch.empty(rows, dtype=torch.float32, device="cuda")
    lse = torch.empty(rows, dtype=torch.float32, device="cuda")
    ctx.extended_logits(d_H, rows_per_seq, d_E, d_W, am, mx, lse, None)
    torch.cuda.synchronize()
    print(f"  extended_logits done {time.time() - t0:.1f}s", flush=True)
    am_h, mx_h, lse_h = am.cpu().numpy(), mx.cpu().numpy(), lse.cpu().numpy()
    # properties that hold at any size, on every row
    assert np.isfinite(mx_h).all() and np.isfinite(lse_h).all()
    assert (lse_h >= mx_h - 1e-4).all()
    size = ctx.codebook()[2].cpu().numpy()
    for b in range(cfg["B"]):
        sl = slice(b * rows_per_seq, (b + 1) * rows_per_seq)
        assert (am_h[sl] >= 0).all() and (am_h[sl] < cfg["V"] + size[b]).all()
        assert (lse_h[sl] <= mx_h[sl] + np.log(cfg["V"] + size[b]) + 1e-3).all()
    # sampled rows, all columns, against the oracle (only sequences whose W_hyper reference was built)
    sub = wl.scaled(cfg, B=cfg["B"])
    rows_s = wl.sample_rows(sub, rows_per_seq, per_seq)
    for b in seqs:
        pick = rows_s[(rows_s // rows_per_seq) == b]
        r = oracle.extended_logits(H[pick], E, refW[b], len(ref[b][1]), cfg["dtype"], return_logits=True)
        errs = check_logits_rows(r, am_h[pick], mx_h[pick], lse_h[pick], None)
        print(f"  seq {b}: {len(pick)} sampled rows, errors {errs}  {time.time() - t0:.1f}s", flush=True)
    ctx.close()


@pytest.mark.parametrize("rows_per_seq", [2, 5, 40])
def test_full_size_few_rows_per_sequence_c3(rows_per_seq):
    """Config 3's codebooks with a few hidden rows per sequence (a verification step of several drafted codes, a
    chunk of a prefill): the tile kernels with short strips and the few-row-tile workgroup mapping.  Sampled rows
    over all columns against the oracle, size-independent properties on every row."""
    import torch

    cfg = wl.CONFIGS["c3"]
    t0 = time.time()
    print(f"[case] full size c3 codebooks, {rows_per_seq} rows per sequence", flush=True)
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    B = cfg["B"]
    rows = B * rows_per_seq
    H = wl.make_hidden(cfg, rows)
    ctx, w = _make_ctx(cfg)
    ref = _encode(ctx, cfg, tokens)
    d_E, d_W = _embed_gpu(ctx, cfg, E)
    seqs = [0, 17, B - 1]
    refW, worst = _check_embed(cfg, ref, E, d_W, w, seqs=seqs)
    d_H = torch_storage(H, cfg["dtype"])
    am = torch.empty(rows, dtype=torch.int32, device="cuda")
    mx = torch.empty(rows, dtype=torch.float32, device="cuda")
    lse = torch.empty(rows, dtype=torch.float32, device="cuda")
    ctx.extended_logits(d_H, rows_per_seq, d_E, d_W, am, mx, lse, None)
    torch.cuda.synchronize()
    am_h, mx_h, lse_h = am.cpu().numpy(), mx.cpu().numpy(), lse.cpu().numpy()
    assert np.isfinite(mx_h).all() and np.isfinite(lse_h).all() and (lse_h >= mx_h - 1e-4).all()
    size = ctx.codebook()[2].cpu().numpy()
    for b in range(B):
        sl = slice(b * rows_per_seq, (b + 1) * rows_per_seq)
        assert (am_h[sl] >= 0).all() and (am_h[sl] < cfg["V"] + size[b]).all()
        assert (lse_h[sl] <= mx_h[sl] + np.log(cfg["V"] + size[b]) + 1e-3).all()
    for b in seqs:
        pick = np.arange(b * rows_per_seq, (b + 1) * rows_per_seq)[[0, rows_per_seq - 1]]
        r = oracle.extended_logits(H[pick], E, refW[b], len(ref[b][1]), cfg["dtype"], return_logits=True)
        errs = check_logits_rows(r, am_h[pick], mx_h[pick], lse_h[pick], None)
        print(f"  seq {b}: first and last row, errors {errs}  {time.time() - t0:.1f}s", flush=True)
    ctx.close()


def test_full_size_decode_step_c3():
    """Config 3: 64 sequences with an 8192-token history, one code per sequence, one hidden row each."""
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.CONFIGS["c3"]
    t0 = time.time()
    print("[case] full size decode step c3", flush=True)
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    B = cfg["B"]
    H = wl.make_hidden(cfg, B)
    ctx, w = _make_ctx(cfg)
    streams = [oracle.LZWStream(cfg["V"], cfg["M"], cfg["cap"]) for _ in range(B)]
    for b in range(B):
        streams[b].encode_chunk(tokens[b].tolist())
    gpu_encode(ctx, tokens, None)
    d_E, d_W = _embed_gpu(ctx, cfg, E)
    print(f"  history encoded and embedded {time.time() - t0:.1f}s", flush=True)
    # one decode step: new code -> codebook update -> embed the new entry -> logits
    sizes = np.array([len(s.entries) for s in streams])
    new = wl.make_step_codes(cfg, sizes, 0)
    d_new = torch.from_numpy(new.reshape(B, 1)).cuda()
    n_tok = torch.empty(B, dtype=torch.int32, device="cuda")
    st = torch.empty(B, dtype=torch.int32, device="cuda")
    ctx.lzw_decode(d_new, None, None, n_tok, st, api.APPEND)
    ctx.hyper_embed(d_E, d_W, None, max_new=1)         # at most one new entry per sequence and step
    d_H = torch_storage(H, cfg["dtype"])
    am = torch.empty(B, dtype=torch.int32, device="cuda")
    mx = torch.empty(B, dtype=torch.float32, device="cuda")
    lse = torch.empty(B, dtype=torch.float32, device="cuda")
    ctx.extended_logits(d_H, 1, d_E, d_W, am, mx, lse, None)
    torch.cuda.synchronize()
    print(f"  step done {time.time() - t0:.1f}s", flush=True)
    assert (st.cpu().numpy() == 0).all()
    for b in range(B):
        streams[b].decode_chunk([int(new[b])])
    size = ctx.codebook()[2].cpu().numpy()
    assert size.tolist() == [len(s.entries) for s in streams]
    am_h, mx_h, lse_h = am.cpu().numpy(), mx.cpu().numpy(), lse.cpu().numpy()
    W_host = storage_to_host(d_W, cfg["dtype"])
    for b in [0, 1, 31, 63]:
        Wr = oracle.hyper_embed(E, cfg["dtype"], streams[b].entries, cfg["cap"], cfg["pool"], w)
        got, want = oracle.to_f64(W_host[b], "bf16"), oracle.to_f64(Wr, "bf16")
        bound = hyper_embed_bound(E, "bf16", streams[b].entries, cfg["pool"], w, cfg["cap"])
        assert (np.abs(got - want) <= 2e-2 * bound + 1e-30).all()
        r = oracle.extended_logits(H[b:b + 1], E, Wr, len(streams[b].entries), "bf16")
        errs = check_logits_rows(r, am_h[b:b + 1], mx_h[b:b + 1], lse_h[b:b + 1], None)
        print(f"  seq {b}: C={len(streams[b].entries)} errors {errs}  {time.time() - t0:.1f}s", flush=True)
    ctx.close()


# ---------------------------------------------------------------------------------------------------
# the one-row-per-sequence kernel at awkward shapes: more than one group of 64 rows, a ragged last group,
# vocabularies and capacities that are no multiple of a unit, empty and unequal codebooks, every row checked
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("B,N,V,d,M,cap", [
    (65, 300, 1000, 3072, 3, 300),      # two row groups, the second with one row
    (3, 200, 777, 128, 4, 0),           # no codebook at all
    (130, 400, 513, 3584, 5, 1030),     # three groups; cap spans three hyper units, the last ragged (beyond 128
                                        # rows the base vocabulary goes to the tile kernel, the hyper units stay)
    (140, 100, 400, 256, 3, 0),         # the same split with no codebook at all
    (300, 120, 2000, 512, 3, 100),      # two row tiles of the tile kernel, 300 hyper units
    (1, 5000, 50000, 256, 2, 600),      # one row: up to 4 sequences the base vocabulary runs on dot-product units too
    (2, 900, 3000, 4096, 3, 700),       # two rows, widest d
    (4, 600, 1300, 2560, 4, 300),       # four rows (one codebook empty, one nearly); d no multiple of 512
    (3, 500, 513, 1024, 3, 1030),       # three rows; V one row past two units, cap spans three hyper units
    (64, 64, 300, 4096, 3, 512),        # widest d the kernel takes
])
def test_decode_kernel_small_shapes_every_row(B, N, V, d, M, cap):
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c3"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=B * 1000 + V)
    print(f"[case] decode kernel B={B} N={N} V={V} d={d} M={M} cap={cap}", flush=True)
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg)
    if B > 2:
        lens[1] = 0                     # an empty codebook next to full ones
        lens[2] = min(N, 7)
    E = wl.make_embeddings(cfg)
    H = wl.make_hidden(cfg, B)
    ctx, w = _make_ctx(cfg)
    ref = _encode(ctx, cfg, tokens, lens)
    d_E, d_W = _embed_gpu(ctx, cfg, E)
    d_H = torch_storage(H, cfg["dtype"])
    am = torch.empty(B, dtype=torch.int32, device="cuda")
    mx = torch.empty(B, dtype=torch.float32, device="cuda")
    lse = torch.empty(B, dtype=torch.float32, device="cuda")
    outs = {}
    for kern in (0, 1):                 # 0: the decode kernel; 1: the general tile kernel on the same call
        ctx.set_option(api.OPT_DECODE_KERNEL, kern)
        ctx.extended_logits(d_H, 1, d_E, d_W, am, mx, lse, None)
        torch.cuda.synchronize()
        outs[kern] = (am.cpu().numpy().copy(), mx.cpu().numpy().copy(), lse.cpu().numpy().copy(), None)
    # the decode kernel also writes the full logits when asked to
    ctx.set_option(api.OPT_DECODE_KERNEL, 0)
    full = torch.full((B, V + cap), 7.0, dtype=torch.float32, device="cuda")
    ctx.extended_logits(d_H, 1, d_E, d_W, am, mx, lse, full)
    torch.cuda.synchronize()
    outs[2] = (am.cpu().numpy().copy(), mx.cpu().numpy().copy(), lse.cpu().numpy().copy(), full.cpu().numpy())
    for b in range(B):
        Wr = oracle.hyper_embed(E, cfg["dtype"], ref[b][1], cap, cfg["pool"], w)
        r = oracle.extended_logits(H[b:b + 1], E, Wr, len(ref[b][1]), cfg["dtype"], return_logits=True)
        for kern in (0, 1, 2):
            a_, m_, l_, f_ = outs[kern]
            check_logits_rows(r, a_[b:b + 1], m_[b:b + 1], l_[b:b + 1], None if f_ is None else f_[b:b + 1], V=V)
    ctx.close()


# ---------------------------------------------------------------------------------------------------
# the generation loop (section 2.3, steps 7-10): pick -> codebook update -> embed the new entry -> logits,
# with each step's pick fed back as the next step's code on the device; eagerly against the oracle, and
# captured once in a HIP graph whose replays must reproduce the eager run
# ---------------------------------------------------------------------------------------------------
def test_feedback_loop_eager_vs_oracle_and_graph_replays():
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c3"], B=6, N=400, V=2000, d=256, cap=300, seed=4242)
    B, V, M, cap, d = (cfg[k] for k in ("B", "V", "M", "cap", "d"))
    K = 12                                            # steps per graph; two replays = 24 steps
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    H_steps = [wl.make_hidden(wl.scaled(cfg, seed=cfg["seed"] + 10 * t), B) for t in range(K)]
    d_H = [torch_storage(h, "bf16") for h in H_steps]
    print("[case] feedback loop, eager and graph", flush=True)

    def fresh():
        ctx, w = _make_ctx(cfg)
        gpu_encode(ctx, tokens, None)
        d_E, d_W = _embed_gpu(ctx, cfg, E)
        return ctx, w, d_E, d_W

    def make_bufs(n):
        return (torch.zeros((n, B), dtype=torch.int32, device="cuda"), torch.zeros((n, B), dtype=torch.float32, device="cuda"),
                torch.zeros((n, B), dtype=torch.float32, device="cuda"), torch.zeros(B, dtype=torch.int32, device="cuda"),
                torch.zeros(B, dtype=torch.int32, device="cuda"))

    def step(ctx, d_E, d_W, bufs, t, slot):
        am, mx, lse, ntok, st = bufs
        ctx.extended_logits(d_H[t % K], 1, d_E, d_W, am[slot], mx[slot], lse[slot], None)
        ctx.lzw_decode(am[slot], None, None, ntok, st, api.APPEND, stride=1)     # the pick is the next code
        ctx.hyper_embed(d_E, d_W, None, max_new=1)

    # ---- eager, 2K steps, checked against the oracle step by step (the oracle is fed the GPU's picks) ----
    ctx, w, d_E, d_W = fresh()
    bufs = make_bufs(2 * K)
    streams = [oracle.LZWStream(V, M, cap) for _ in range(B)]
    for b in range(B):
        streams[b].encode_chunk(tokens[b].tolist())
    for t in range(2 * K):
        step(ctx, d_E, d_W, bufs, t, t)
        torch.cuda.synchronize()
        assert int(bufs[4].abs().sum()) == 0
        am_h, mx_h, lse_h = bufs[0][t].cpu().numpy(), bufs[1][t].cpu().numpy(), bufs[2][t].cpu().numpy()
        for b in range(B):
            Wr = oracle.hyper_embed(E, "bf16", streams[b].entries, cap, cfg["pool"], w)
            r = oracle.extended_logits(H_steps[t % K][b:b + 1], E, Wr, len(streams[b].entries), "bf16", return_logits=True)
            check_logits_rows(r, am_h[b:b + 1], mx_h[b:b + 1], lse_h[b:b + 1], None)
            _, rst = streams[b].decode_chunk([int(am_h[b])])
            assert rst == 0
        size = ctx.codebook()[2].cpu().numpy()
        assert size.tolist() == [len(s.entries) for s in streams], f"step {t}"
    eager_am = bufs[0].cpu().numpy()
    eager_W = d_W.clone()
    eager_size = ctx.codebook()[2].cpu().numpy().copy()
    assert (eager_size > 0).all()
    ctx.close()

    # ---- the same K steps captured once, replayed twice, unrelated eager work in between ----------------
    ctx, w, d_E, d_W = fresh()
    gbufs = make_bufs(K)
    warm = make_bufs(1)
    ctx.extended_logits(d_H[0], 1, d_E, d_W, warm[0][0], warm[1][0], warm[2][0], None)   # sizes the library's scratch
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for t in range(K):
            step(ctx, d_E, d_W, gbufs, t, t)
    for rep in range(2):
        graph.replay()
        torch.cuda.synchronize()
        got = gbufs[0].cpu().numpy()
        assert (got == eager_am[rep * K:(rep + 1) * K]).all(), f"replay {rep}: picks differ from the eager run"
        assert int(gbufs[4].abs().sum()) == 0
        junk = torch.randn(1 << 20, device="cuda").sum().item()                        # eager work between replays
        assert np.isfinite(junk)
    assert (ctx.codebook()[2].cpu().numpy() == eager_size).all()
    assert torch.equal(d_W, eager_W)
    ctx.close()
