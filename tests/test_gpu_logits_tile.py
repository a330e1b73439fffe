"""GPU parity of the bf16 MFMA tile kernels of extended_logits (base part and per-sequence hyper part), the
kernels the prefill benchmark times: every row and, through planted rows, every column.

A call lands on those kernels when the context is bf16, d is a multiple of 64, there are several hidden rows
per sequence and no full-logits output is asked for; each test checks the library's launch counters to make
sure that is where its calls went.  Joint logits, one softmax over base and hyper vocabulary, the pick:
section 2.3, steps 7-9; every position of a sequence sees the sequence's final codebook (section 2.4).

Bars as for the other logits tests: max and lse within 2e-2 * max(1, |ref|), argmax identical wherever the
oracle's two largest logits differ by more than 1e-2 (elsewhere it must name a logit within that gap).
"""
import time

import numpy as np
import pytest

import oracle
from paper_2506_01084_amd import workloads as wl

from helpers import check_logits_rows, gpu_encode, oracle_encode_batch, storage_to_host, torch_storage

pytestmark = pytest.mark.gpu


def _map(lr, ls, xr, xs):
    return lr | (ls << 8) | (xr << 16) | (xs << 24)


# (strip, map) settings every small case runs under: automatic; one tile per workgroup; strips of three with
# the XCDs side by side along the rows; two-tile row blocks with a 2 x 4 XCD split
SETTINGS = [(0, 0), (1, 0), (3, _map(1, 3, 8, 1)), (2, _map(2, 1, 2, 4)), (0, _map(4, 8, 4, 2))]


def _ctx(cfg):
    from paper_2506_01084_amd import api

    return api.Context(B=cfg["B"], V=cfg["V"], M=cfg["M"], cap=cfg["cap"], d=cfg["d"], dtype="bf16", pool=cfg["pool"],
                       w=wl.make_pool_weights(cfg).tolist())


def _run(ctx, d_H, rows_per_seq, d_Wb, d_Wh, strip, mapping):
    """One extended_logits call that must run on the tile kernels; returns host (argmax, max, lse)."""
    import torch
    from paper_2506_01084_amd import api

    rows = d_H.shape[0]
    am = torch.full((rows,), -5, dtype=torch.int32, device="cuda")
    mx = torch.full((rows,), 777.0, dtype=torch.float32, device="cuda")
    lse = torch.full((rows,), 777.0, dtype=torch.float32, device="cuda")
    ctx.set_option(api.OPT_LOGITS_KERNEL, 4)     # the tile kernel also where few rows would go to the streaming kernel
    ctx.set_option(api.OPT_LOGITS_STRIP, strip)
    ctx.set_option(api.OPT_LOGITS_MAP, mapping)
    before = ctx.read_launches()
    ctx.extended_logits(d_H, rows_per_seq, d_Wb, d_Wh, am, mx, lse, None)
    torch.cuda.synchronize()
    after = ctx.read_launches()
    assert after["tile_base"] == before["tile_base"] + 1, "the base part did not run on the MFMA tile kernel"
    assert after["tile_hyper"] == before["tile_hyper"] + (1 if ctx.cap > 0 else 0), "hyper part not on the tile kernel"
    assert after["general"] == before["general"] and after["decode"] == before["decode"]
    return am.cpu().numpy(), mx.cpu().numpy(), lse.cpu().numpy()


# ---------------------------------------------------------------------------------------------------
# ragged shapes: V, cap, rows and rows per sequence no multiples of the 256-wide tile, one to nine K slabs,
# unequal codebooks (one empty, one nearly empty, full ones), W_hyper from hyper_embed; every row
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("B,rows_per_seq,V,d,M,cap,pool", [
    (3, 300, 1000, 128, 3, 300, "mean"),        # rows/sequence spans two row tiles, cap two weight tiles
    (2, 517, 2500, 256, 4, 700, "weighted"),    # ten base tiles: strips of 4, 4, 2
    (5, 70, 600, 64, 5, 130, "mean"),           # one K slab per tile: the stream crosses a tile every slab
    (4, 260, 1300, 320, 3, 513, "mean"),        # five slabs (odd: the two LDS stages swap roles per tile)
    (1, 1000, 777, 192, 2, 0, "mean"),          # no hyper vocabulary
    (9, 33, 300, 576, 3, 257, "mean"),          # nine slabs, 297 rows, cap one column past a tile
    (2, 100, 1300, 320, 3, 300, "mean"),        # 200 rows, a single row tile: the weight tiles walk K from different slabs
    (1, 250, 2100, 192, 3, 0, "mean"),          # the same with three slabs and nine weight tiles (every start, wrapping round)
])
def test_tile_kernels_every_row_ragged(B, rows_per_seq, V, d, M, cap, pool):
    import torch

    N = 900
    cfg = dict(name="tile", B=B, N=N, V=V, d=d, dtype="bf16", M=M, cap=cap, zipf_s=1.2, copy_frac=0.4, span=(2, 7),
               mode="motif", pool=pool, seed=9000 + V + d)
    print(f"[case] tile kernels B={B} rows/seq={rows_per_seq} V={V} d={d} M={M} cap={cap} {pool}", flush=True)
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg)
    if B > 2:
        lens[1] = 0                      # an empty codebook beside full ones
        lens[2] = 9                      # and one with a handful of entries
    E = wl.make_embeddings(cfg)
    rows = B * rows_per_seq
    H = wl.make_hidden(cfg, rows)
    w = wl.make_pool_weights(cfg)
    ctx = _ctx(cfg)
    gpu_encode(ctx, tokens, lens)
    ref = oracle_encode_batch(tokens, lens, V, M, cap)
    d_E = torch_storage(E, "bf16")
    d_W = torch.full((B, cap, d), 1.0, dtype=torch.bfloat16, device="cuda")
    if cap:
        ctx.hyper_embed(d_E, d_W)
        torch.cuda.synchronize()
    sizes = [len(r[1]) for r in ref]
    print(f"  codebook sizes {sizes}", flush=True)
    if cap and B > 2:
        assert sizes[1] == 0 and max(sizes) == cap
    d_H = torch_storage(H, "bf16")
    want = []
    for b in range(B):
        Wr = oracle.hyper_embed(E, "bf16", ref[b][1], cap, pool, w) if cap else np.zeros((0, d), np.uint16)
        want.append(oracle.extended_logits(H[b * rows_per_seq:(b + 1) * rows_per_seq], E, Wr, sizes[b], "bf16"))
    for strip, mapping in SETTINGS:
        am, mx, lse = _run(ctx, d_H, rows_per_seq, d_E, d_W, strip, mapping)
        worst = dict(max=0.0, lse=0.0)
        for b in range(B):
            sl = slice(b * rows_per_seq, (b + 1) * rows_per_seq)
            errs = check_logits_rows(want[b], am[sl], mx[sl], lse[sl], None)
            worst = {k: max(worst[k], errs[k]) for k in worst}
        print(f"  strip {strip} map {mapping:#x}: every row ok, worst {worst}", flush=True)
    ctx.close()


# ---------------------------------------------------------------------------------------------------
# planted rows: for every existing column v of a sequence (base and hyper) one hidden row is 64 x that
# column's weight row (exact in bf16), so the oracle's pick for the row is v with a wide gap: a column that
# lands in the wrong place anywhere between the LDS layout, the MFMA lane map and the fold moves a pick
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("B,V,d,cap", [
    (2, 700, 128, 300),
    (2, 2300, 192, 520),                        # nine base tiles (strips 4, 4, 1), three hyper tiles
])
def test_tile_kernels_planted_rows_pin_every_column(B, V, d, cap):
    import torch

    M, N = 3, 1200
    cfg = dict(name="plant", B=B, N=N, V=V, d=d, dtype="bf16", M=M, cap=cap, zipf_s=1.1, copy_frac=0.4, span=(2, 6),
               mode="motif", pool="mean", seed=7100 + V)
    print(f"[case] planted rows B={B} V={V} d={d} cap={cap}", flush=True)
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg)
    lens[1] = 300                         # a codebook that stops short of cap: its last columns do not exist
    ctx = _ctx(cfg)
    gpu_encode(ctx, tokens, lens)
    sizes = [len(r[1]) for r in oracle_encode_batch(tokens, lens, V, M, cap)]
    assert sizes[0] == cap and 0 < sizes[1] < cap, sizes
    Wb = wl.make_embeddings(cfg)                                                  # [V, d] N(0, 0.02)
    # W_hyper is the caller's buffer: independent random rows here (pooled rows would tie with their own
    # constituents' base rows), unused slots included -- those must never be picked
    Wh = wl.normal_matrix(cfg["seed"] + 50, B * cap, d, 0.02, "bf16").reshape(B, cap, d)
    rows_per_seq = V + cap
    H = wl.make_hidden(cfg, B * rows_per_seq)                                     # rows that plant nothing stay random
    rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 60))
    planted = np.full(B * rows_per_seq, -1, dtype=np.int64)
    for b in range(B):
        n_cols = V + sizes[b]
        where = b * rows_per_seq + rng.permutation(rows_per_seq)[:n_cols]         # column v -> a scattered row
        Wcat = np.concatenate([Wb, Wh[b, :sizes[b]]], axis=0)
        H[where] = oracle.round_to_storage(64.0 * oracle.to_f64(Wcat, "bf16"), "bf16")
        planted[where] = np.arange(n_cols)
    want = [oracle.extended_logits(H[b * rows_per_seq:(b + 1) * rows_per_seq], Wb, Wh[b], sizes[b], "bf16")
            for b in range(B)]
    for b in range(B):                    # the plant works in the oracle: pick = planted column, gap wide
        p = planted[b * rows_per_seq:(b + 1) * rows_per_seq]
        has = p >= 0
        assert (want[b]["argmax"][has] == p[has]).all()
        assert (want[b]["margin"][has] > 0.5).all(), want[b]["margin"][has].min()
    d_H, d_Wb, d_Wh = torch_storage(H, "bf16"), torch_storage(Wb, "bf16"), torch_storage(Wh, "bf16")
    for strip, mapping in SETTINGS:
        am, mx, lse = _run(ctx, d_H, rows_per_seq, d_Wb, d_Wh, strip, mapping)
        has = planted >= 0
        wrong = np.nonzero(has & (am != planted))[0]
        assert wrong.size == 0, f"strip {strip} map {mapping:#x}: rows {wrong[:8]} pick {am[wrong[:8]]}, planted {planted[wrong[:8]]}"
        for b in range(B):
            sl = slice(b * rows_per_seq, (b + 1) * rows_per_seq)
            check_logits_rows(want[b], am[sl], mx[sl], lse[sl], None)
        print(f"  strip {strip} map {mapping:#x}: {int(has.sum())} planted columns picked, every row ok", flush=True)
    ctx.close()


# ---------------------------------------------------------------------------------------------------
# full benchmark size, the launch configuration the benchmark times: 256 sampled rows of two sequences that
# hit every row position of a 256-row tile once, all columns against the oracle
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["c2", "c4", "c5"])
def test_full_size_every_row_position_of_a_tile(name):
    import torch

    cfg = wl.CONFIGS[name]
    t0 = time.time()
    print(f"[case] full size {name}: one sampled row per row position of a tile", flush=True)
    B, N, V, d, M, cap = (cfg[k] for k in ("B", "N", "V", "d", "M", "cap"))
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    rows = B * N
    H = wl.make_hidden(cfg, rows)
    w = wl.make_pool_weights(cfg)
    ctx = _ctx(cfg)
    gpu_encode(ctx, tokens, None)
    ref = oracle_encode_batch(tokens, wl.make_lens(cfg), V, M, cap)
    d_E = torch_storage(E, "bf16")
    d_W = torch.empty((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.hyper_embed(d_E, d_W)
    d_H = torch_storage(H, "bf16")
    am, mx, lse = _run(ctx, d_H, N, d_E, d_W, 0, 0)
    print(f"  extended_logits done {time.time() - t0:.1f}s", flush=True)
    rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 6))
    W_host = storage_to_host(d_W, "bf16")
    for b, positions in ((0, np.arange(0, 128)), (B - 1, np.arange(128, 256))):
        tiles = rng.integers(0, N // 256, size=positions.size)
        pick = b * N + tiles * 256 + positions            # (b * N is a multiple of 256: position = row % 256)
        Wr = oracle.hyper_embed(E, "bf16", ref[b][1], cap, cfg["pool"], w)
        assert (W_host[b] == Wr).mean() > 0.99           # (the embedding itself is checked elsewhere)
        r = oracle.extended_logits(H[pick], E, Wr, len(ref[b][1]), "bf16", return_logits=True)
        errs = check_logits_rows(r, am[pick], mx[pick], lse[pick], None)
        print(f"  seq {b}: {pick.size} rows, errors {errs}  {time.time() - t0:.1f}s", flush=True)
    ctx.close()


# ---------------------------------------------------------------------------------------------------
# 2..64 hidden rows per sequence: the hyper part runs on the decode kernel's per-sequence units (one workgroup
# per sequence and 256 rows of its W_hyper: dot-product units with the hidden rows in registers up to 4 rows per
# sequence, matrix-core units beyond), the base vocabulary on the streaming or the tile kernel; every row
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("B,rows_per_seq,V,d,M,cap,pool", [
    (5, 2, 1000, 128, 3, 300, "mean"),          # two rows per sequence, cap spans two blocks of 256
    (7, 3, 900, 512, 3, 520, "mean"),           # three rows per sequence; cap ends 8 rows into a third block
    (6, 4, 1500, 4096, 4, 300, "weighted"),     # four rows per sequence (the most the dot-product units take), widest rows
    (4, 2, 800, 2560, 3, 257, "mean"),          # d no multiple of 512: lanes whose last chunk lies past the row end
    (4, 17, 700, 256, 4, 1030, "weighted"),     # one row past a 16-row group; five blocks, the last with 6 rows
    (70, 5, 520, 384, 3, 257, "mean"),          # 350 rows: two row tiles of the base part; cap one past a block
    (3, 64, 300, 1024, 5, 100, "mean"),         # the most rows per sequence this path takes; one full K phase
    (6, 33, 2000, 4096, 3, 64, "mean"),         # widest rows: four K phases
])
def test_few_rows_per_sequence_every_row(B, rows_per_seq, V, d, M, cap, pool):
    import torch
    from paper_2506_01084_amd import api

    N = 2400
    cfg = dict(name="few", B=B, N=N, V=V, d=d, dtype="bf16", M=M, cap=cap, zipf_s=1.2, copy_frac=0.4, span=(2, 7),
               mode="motif", pool=pool, seed=9900 + V + d)
    print(f"[case] few rows per sequence B={B} rows/seq={rows_per_seq} V={V} d={d} M={M} cap={cap} {pool}", flush=True)
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg)
    lens[1] = 0                          # an empty codebook
    lens[2] = 9                          # a handful of entries
    if B > 3:
        lens[3] = 300                    # a codebook that ends inside a block
    E = wl.make_embeddings(cfg)
    rows = B * rows_per_seq
    H = wl.make_hidden(cfg, rows)
    w = wl.make_pool_weights(cfg)
    ctx = _ctx(cfg)
    gpu_encode(ctx, tokens, lens)
    ref = oracle_encode_batch(tokens, lens, V, M, cap)
    sizes = [len(r[1]) for r in ref]
    print(f"  codebook sizes {sizes[:8]}", flush=True)
    assert sizes[1] == 0 and max(sizes) == cap
    d_E = torch_storage(E, "bf16")
    d_W = torch.full((B, cap, d), 1.0, dtype=torch.bfloat16, device="cuda")      # unused slots hold ones
    ctx.hyper_embed(d_E, d_W)
    d_Wp = d_W.clone()
    for b in range(B):
        d_Wp[b, sizes[b]:] = 900.0       # rows that do not exist must never be read into a result
    d_H = torch_storage(H, "bf16")
    am = torch.full((rows,), -5, dtype=torch.int32, device="cuda")
    mx = torch.full((rows,), 777.0, dtype=torch.float32, device="cuda")
    lse = torch.full((rows,), 777.0, dtype=torch.float32, device="cuda")
    before = ctx.read_launches()
    ctx.extended_logits(d_H, rows_per_seq, d_E, d_Wp, am, mx, lse, None)
    torch.cuda.synchronize()
    after = ctx.read_launches()
    # hyper part: the per-sequence units of the decode kernel.  Base part: up to 192 rows in all the weight-streaming
    # kernel, beyond that the tile kernel
    want_mid = 1 if rows <= 192 else 0
    want_tile = 1 if rows > 192 else 0
    assert after["decode"] == before["decode"] + 1 and after["mid"] == before["mid"] + want_mid
    assert after["tile_base"] == before["tile_base"] + want_tile and after["tile_hyper"] == before["tile_hyper"]
    assert after["general"] == before["general"]
    am_h, mx_h, lse_h = am.cpu().numpy(), mx.cpu().numpy(), lse.cpu().numpy()
    worst = dict(max=0.0, lse=0.0)
    for b in range(B):
        Wr = oracle.hyper_embed(E, "bf16", ref[b][1], cap, pool, w)
        sl = slice(b * rows_per_seq, (b + 1) * rows_per_seq)
        r = oracle.extended_logits(H[sl], E, Wr, sizes[b], "bf16")
        errs = check_logits_rows(r, am_h[sl], mx_h[sl], lse_h[sl], None)
        worst = {k: max(worst[k], errs[k]) for k in worst}
    print(f"  every row ok, worst {worst}", flush=True)
    # the tile kernels on the same call give the same picks
    ctx.set_option(api.OPT_DECODE_KERNEL, 1)
    ctx.set_option(api.OPT_LOGITS_KERNEL, 4)
    am2, mx2, lse2 = torch.empty_like(am), torch.empty_like(mx), torch.empty_like(lse)
    ctx.extended_logits(d_H, rows_per_seq, d_E, d_Wp, am2, mx2, lse2, None)
    torch.cuda.synchronize()
    assert ctx.read_launches()["tile_hyper"] == after["tile_hyper"] + 1
    assert ctx.read_launches()["tile_base"] == after["tile_base"] + 1
    am2_h, mx2_h, lse2_h = am2.cpu().numpy(), mx2.cpu().numpy(), lse2.cpu().numpy()
    for b in range(B):
        Wr = oracle.hyper_embed(E, "bf16", ref[b][1], cap, pool, w)
        sl = slice(b * rows_per_seq, (b + 1) * rows_per_seq)
        check_logits_rows(oracle.extended_logits(H[sl], E, Wr, sizes[b], "bf16"), am2_h[sl], mx2_h[sl], lse2_h[sl], None)
    # (picks may differ between the two kernels only where two logits tie within rounding -- a pooled row of a
    # repeated token equals that token's base row; both were held to the oracle's margin rule above)
    check_rows = (am != am2).cpu().numpy()
    assert check_rows.mean() < 0.05
    assert torch.allclose(mx, mx2, rtol=1e-4, atol=1e-4) and torch.allclose(lse, lse2, rtol=1e-4, atol=1e-4)
    ctx.close()


def test_few_rows_per_sequence_planted_hyper_columns():
    """Planted rows for the matrix-core hyper units: every existing hyper column of every sequence is the pick of
    one hidden row of that sequence (64 rows per sequence, 64 columns planted per call, several calls)."""
    import torch

    B, V, d, cap, M, rps = 3, 400, 256, 600, 3, 64
    cfg = dict(name="plant2", B=B, N=2000, V=V, d=d, dtype="bf16", M=M, cap=cap, zipf_s=1.1, copy_frac=0.4, span=(2, 6),
               mode="motif", pool="mean", seed=7300)
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg)
    lens[1] = 500
    ctx = _ctx(cfg)
    gpu_encode(ctx, tokens, lens)
    sizes = [len(r[1]) for r in oracle_encode_batch(tokens, lens, V, M, cap)]
    assert sizes[0] == cap and 0 < sizes[1] < cap
    Wb = wl.make_embeddings(cfg)
    Wh = wl.normal_matrix(cfg["seed"] + 50, B * cap, d, 0.02, "bf16").reshape(B, cap, d)
    d_Wb, d_Wh = torch_storage(Wb, "bf16"), torch_storage(Wh, "bf16")
    rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 60))
    n_calls = (cap + rps - 1) // rps
    for call in range(n_calls):
        H = wl.make_hidden(wl.scaled(cfg, seed=cfg["seed"] + call), B * rps)
        planted = np.full(B * rps, -1, dtype=np.int64)
        for b in range(B):
            cols = np.arange(call * rps, min((call + 1) * rps, sizes[b]))
            where = b * rps + rng.permutation(rps)[:cols.size]
            H[where] = oracle.round_to_storage(64.0 * oracle.to_f64(Wh[b, cols], "bf16"), "bf16")
            planted[where] = V + cols
        am = torch.empty(B * rps, dtype=torch.int32, device="cuda")
        mx = torch.empty(B * rps, dtype=torch.float32, device="cuda")
        lse = torch.empty(B * rps, dtype=torch.float32, device="cuda")
        before = ctx.read_launches()["decode"]
        ctx.extended_logits(torch_storage(H, "bf16"), rps, d_Wb, d_Wh, am, mx, lse, None)
        torch.cuda.synchronize()
        assert ctx.read_launches()["decode"] == before + 1
        am_h, mx_h, lse_h = am.cpu().numpy(), mx.cpu().numpy(), lse.cpu().numpy()
        for b in range(B):
            sl = slice(b * rps, (b + 1) * rps)
            r = oracle.extended_logits(H[sl], Wb, Wh[b], sizes[b], "bf16")
            has = planted[sl] >= 0
            assert (r["argmax"][has] == planted[sl][has]).all() and (r["margin"][has] > 0.5).all()
            assert (am_h[sl][has] == planted[sl][has]).all(), f"call {call} seq {b}"
            check_logits_rows(r, am_h[sl], mx_h[sl], lse_h[sl], None)
    ctx.close()
