"""GPU parity: extended_sample (temperature sampling from the joint softmax, section 2.3 steps 8-9) through
the C ABI against the float64 oracle, which draws the same Philox numbers from its own implementation.

Bars: the drawn column is identical wherever the oracle's two largest perturbed values are more than 1e-3
apart (float32 logits and float32 noise against float64 ones); closer than that, the GPU's column must be one
of those near-maximal ones.  The reported log-probability is within 2e-2 * max(1, |ref|) of the oracle's value
for that column.
"""
import numpy as np
import pytest

import oracle
from oracle import sampling
from paper_2506_01084_amd import workloads as wl

from helpers import gpu_encode, oracle_encode_batch, storage_to_host, torch_storage

pytestmark = pytest.mark.gpu

GAP = 1e-3


def _check_draws(ref, tok, lp, T):
    """ref: oracle.extended_sample result for the rows of one sequence; tok, lp: the GPU's, same rows."""
    for i in range(len(tok)):
        z = ref["logits"][i] / T
        pert = sampling.sample_row(ref["logits"][i], T, *ref["coords"][i])["perturbed"]
        if ref["gap"][i] > GAP:
            assert tok[i] == ref["token"][i], f"row {i}: drew {tok[i]}, oracle {ref['token'][i]} (gap {ref['gap'][i]})"
        else:
            assert pert.max() - pert[tok[i]] <= GAP + 1e-6
        m = z.max()
        want = z[tok[i]] - (m + np.log(np.exp(z - m).sum()))
        assert abs(lp[i] - want) <= 2e-2 * max(1.0, abs(want)), (i, lp[i], want)


def _setup(cfg, lens=None):
    import torch
    from paper_2506_01084_amd import api

    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg) if lens is None else lens
    E = wl.make_embeddings(cfg)
    H = wl.make_hidden(cfg, cfg["B"])
    w = wl.make_pool_weights(cfg)
    ctx = api.Context(B=cfg["B"], V=cfg["V"], M=cfg["M"], cap=cfg["cap"], d=cfg["d"], dtype=cfg["dtype"],
                      pool=cfg["pool"], w=w.tolist())
    gpu_encode(ctx, tokens, lens)
    ref = oracle_encode_batch(tokens, lens, cfg["V"], cfg["M"], cfg["cap"])
    d_E = torch_storage(E, cfg["dtype"])
    d_W = torch.zeros((cfg["B"], cfg["cap"], cfg["d"]), dtype=ctx.torch_dtype, device="cuda")
    ctx.hyper_embed(d_E, d_W)
    d_H = torch_storage(H, cfg["dtype"])
    torch.cuda.synchronize()
    return ctx, ref, E, H, w, d_E, d_W, d_H


@pytest.mark.parametrize("B,N,V,d,M,cap", [
    (65, 300, 1000, 256, 3, 300),
    (128, 120, 1301, 384, 3, 70),           # 128 rows: the base vocabulary on the weight-streaming kernel, 6 K slabs
    (5, 200, 777, 128, 4, 0),
    (130, 400, 513, 384, 5, 1030),      # 129..192 rows: the streaming kernel's widest build (base), hyper units
    (230, 100, 1500, 384, 3, 50),       # 193..256 rows: the draw folded into the tile kernel, one row tile (rotated K walk)
    (300, 150, 2300, 256, 3, 90),       # two row tiles, ragged column tail, every sequence one hyper unit
    (140, 100, 700, 128, 3, 0),         # 140 rows with no codebook
    (2, 3000, 40000, 4096, 3, 700),
    (1, 500, 3000, 512, 3, 600),        # up to 4 sequences: the base vocabulary on dot-product units, draw folded in
    (4, 300, 2000, 2560, 3, 513),       # four sequences; d no multiple of 512
    (3, 400, 1300, 1024, 4, 100),
])
def test_draws_match_oracle_every_row(B, N, V, d, M, cap):
    import torch

    cfg = wl.scaled(wl.CONFIGS["c3"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=7 * B + V)
    print(f"[case] sampling B={B} V={V} d={d} cap={cap}", flush=True)
    lens = wl.make_lens(cfg)
    if B > 1:
        lens[1] = 0
    ctx, ref, E, H, w, d_E, d_W, d_H = _setup(cfg, lens)
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    lp = torch.empty(B, dtype=torch.float32, device="cuda")
    for T, seed, step in ((1.0, 1234, 0), (0.6, (77 << 32) | 5, (3 << 32) | 9), (1.7, 2**63 + 11, 41)):
        ctx.extended_sample(d_H, 1, d_E, d_W, T, seed, step, tok, lp)
        torch.cuda.synchronize()
        tok_h, lp_h = tok.cpu().numpy(), lp.cpu().numpy()
        decided = 0
        for b in range(B):
            C = len(ref[b][1])
            Wr = oracle.hyper_embed(E, cfg["dtype"], ref[b][1], cap, cfg["pool"], w)
            r = sampling.extended_sample(H[b:b + 1], E, Wr, C, cfg["dtype"], T, seed, step, row0=b)
            r["coords"] = [(seed, step, b)]
            assert 0 <= tok_h[b] < V + C
            _check_draws(r, tok_h[b:b + 1], lp_h[b:b + 1], T)
            decided += int(r["gap"][0] > GAP)
        assert decided >= 0.9 * B - (1 if B < 8 else 0)           # the comparison is not vacuous
    ctx.close()


def test_cold_draw_is_the_argmax_and_draws_are_reproducible():
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c3"], B=40, N=500, V=3000, d=512, cap=400, seed=99)
    B = cfg["B"]
    ctx, ref, E, H, w, d_E, d_W, d_H = _setup(cfg)
    am = torch.empty(B, dtype=torch.int32, device="cuda")
    mx = torch.empty(B, dtype=torch.float32, device="cuda")
    lse = torch.empty(B, dtype=torch.float32, device="cuda")
    ctx.extended_logits(d_H, 1, d_E, d_W, am, mx, lse, None)
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    lp = torch.empty(B, dtype=torch.float32, device="cuda")
    ctx.extended_sample(d_H, 1, d_E, d_W, 1e-3, 5, 0, tok, lp)          # T -> 0
    torch.cuda.synchronize()
    # the gap between the two best logits is scaled by 1000: noise of a few units cannot bridge it on most rows
    same = (tok == am).float().mean().item()
    assert same > 0.9
    sure = tok == am
    assert (lp[sure] > -0.05).float().mean().item() > 0.9                 # probability close to one there
    assert (lp <= 1e-6).all()
    draws = {}
    for step in (0, 1, 0, 2):
        ctx.extended_sample(d_H, 1, d_E, d_W, 1.0, 5, step, tok, None)    # log-probability output is optional
        torch.cuda.synchronize()
        t = tok.cpu().numpy().copy()
        if step in draws:
            assert (draws[step] == t).all()                               # same coordinates, same draws
        draws[step] = t
    assert (draws[0] != draws[1]).any() and (draws[1] != draws[2]).any()
    # argument checks: temperature, shapes the kernel is not built for
    with pytest.raises(api.Z2ZError):
        ctx.extended_sample(d_H, 1, d_E, d_W, 0.0, 5, 0, tok, None)
    with pytest.raises(api.Z2ZError):
        ctx.extended_sample(d_H, 1, d_E, d_W, float("nan"), 5, 0, tok, None)
    ctx.close()
    c2 = api.Context(B=2, V=100, M=3, cap=10, d=64, dtype="f32")
    h = torch.zeros((2, 64), device="cuda")
    e = torch.zeros((100, 64), device="cuda")
    wh = torch.zeros((2, 10, 64), device="cuda")
    with pytest.raises(api.Z2ZError):
        c2.extended_sample(h, 1, e, wh, 1.0, 1, 0, torch.empty(2, dtype=torch.int32, device="cuda"), None)
    c2.close()


def test_draw_frequencies_follow_the_softmax():
    """Many steps on one small shape: chi-square of the GPU's draws against the oracle's probabilities."""
    import torch

    cfg = wl.scaled(wl.CONFIGS["c3"], B=64, N=100, V=12, d=128, M=2, cap=4, seed=5)
    B, V = cfg["B"], cfg["V"]
    ctx, ref, E, H, w, d_E, d_W, d_H = _setup(cfg)
    T = 0.25                      # the logits of this shape are small; a low temperature spreads the probabilities
    n_steps = 400
    toks = torch.empty((n_steps, B), dtype=torch.int32, device="cuda")
    for s in range(n_steps):
        ctx.extended_sample(d_H, 1, d_E, d_W, T, 2024, s, toks[s], None)
    torch.cuda.synchronize()
    toks_h = toks.cpu().numpy()
    chi2_total, dof = 0.0, 0
    for b in range(0, B, 8):
        C = len(ref[b][1])
        Wr = oracle.hyper_embed(E, cfg["dtype"], ref[b][1], cfg["cap"], cfg["pool"], w)
        lg = oracle.extended_logits(H[b:b + 1], E, Wr, C, cfg["dtype"])["logits"][0] / T
        p = np.exp(lg - lg.max())
        p /= p.sum()
        counts = np.bincount(toks_h[:, b], minlength=V + C)[: V + C]
        assert toks_h[:, b].max() < V + C
        keep = n_steps * p >= 5
        chi2_total += (((counts - n_steps * p) ** 2 / (n_steps * p))[keep]).sum()
        dof += int(keep.sum()) - 1
    # chi-square with `dof` degrees of freedom: mean dof, variance 2 dof; five standard deviations
    assert chi2_total < dof + 5 * np.sqrt(2 * dof), (chi2_total, dof)
    ctx.close()


def test_full_size_decode_step_c3_sampled_sequences():
    import time
    import torch

    cfg = wl.CONFIGS["c3"]
    t0 = time.time()
    print("[case] full size sampling step c3", flush=True)
    ctx, ref, E, H, w, d_E, d_W, d_H = _setup(cfg, np.full(cfg["B"], cfg["N"], dtype=np.int32))
    B = cfg["B"]
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    lp = torch.empty(B, dtype=torch.float32, device="cuda")
    T, seed, step = 0.8, 31337, 123456789012
    ctx.extended_sample(d_H, 1, d_E, d_W, T, seed, step, tok, lp)
    torch.cuda.synchronize()
    tok_h, lp_h = tok.cpu().numpy(), lp.cpu().numpy()
    W_host = storage_to_host(d_W, cfg["dtype"])
    for b in (0, 17, 63):
        C = len(ref[b][1])
        # the GPU's own (already parity-checked) hyper rows: the draw is compared on identical weights
        r = sampling.extended_sample(H[b:b + 1], E, W_host[b], C, cfg["dtype"], T, seed, step, row0=b)
        r["coords"] = [(seed, step, b)]
        _check_draws(r, tok_h[b:b + 1], lp_h[b:b + 1], T)
        print(f"  seq {b}: C={C} token {tok_h[b]} logprob {lp_h[b]:.4f} gap {r['gap'][0]:.4f}  {time.time() - t0:.1f}s", flush=True)
    ctx.close()


# ---------------------------------------------------------------------------------------------------------
# truncation: top-k / nucleus filters in front of the draw
# ---------------------------------------------------------------------------------------------------------
def _check_truncated(logits_row, T, k, p, seed, step, row, tok, lp):
    """The GPU's draw against the oracle's.  Where the oracle's truncation rule came within rounding of keeping
    one column more or fewer (float32 sums and logits against float64 ones), the draws for those neighbouring
    prefixes are accepted too; and where columns at the cut are tied to within rounding (a base token and a
    hypertoken with the same vector get their logits from different kernels, in different summation orders),
    any of the tied columns may be the ones kept.  Returns True when the row was decidable (the perturbed maximum
    stands clear)."""
    r = sampling.sample_row_truncated(logits_row, T, k, p, seed, step, row)
    z = logits_row / T
    order = np.lexsort((np.arange(len(z)), -z))
    pert = r["perturbed"]
    TIE = 1e-4
    sizes = [r["n_kept"]]
    if r["order_gap"] < TIE or r["mass_gap"] < 4e-6:
        sizes += [max(1, r["n_kept"] - 1), min(len(z), r["n_kept"] + 1)]
    if r["gap"] < GAP:
        assert 0 <= tok < len(z) and lp <= 1e-6
        return False
    problems = []
    for n in sizes:
        cut = z[order[n - 1]]
        above = order[z[order] > cut + TIE]                     # kept whatever the order of the tied ones is
        tied = order[np.abs(z[order] - cut) <= TIE]             # n - len(above) of these are kept
        room = n - len(above)
        if tok not in above and tok not in tied:
            problems.append((n, "not among the kept or tied columns"))
            continue
        # tok wins the draw iff nothing kept beats it: everything above must not, and at most len(tied) - room
        # of the tied columns may (those can be the ones left out); tok itself takes one of the `room` places
        if len(above) and pert[above].max() > pert[tok]:
            problems.append((n, "a kept column has a larger perturbed value"))
            continue
        beaten_by = int((pert[tied] > pert[tok]).sum())
        places = room - (1 if tok in tied else 0)
        if len(tied) - beaten_by - (1 if tok in tied else 0) < places:
            problems.append((n, "too many tied columns beat it"))
            continue
        mz = z[order[0]]
        mass = np.exp(z[above] - mz).sum() + room * np.exp(cut - mz)
        want = z[tok] - (mz + np.log(mass))
        if abs(lp - want) <= 2e-2 * max(1.0, abs(want)):
            return True
        problems.append((n, f"log-probability {lp} against {want}"))
    raise AssertionError(f"row {row}: drew {tok}, oracle {r['token']} (kept {r['n_kept']}): {problems}")


@pytest.mark.parametrize("whole_row_only", [0, 1])
@pytest.mark.parametrize("B,N,V,d,M,cap", [
    (65, 300, 1000, 256, 3, 300),
    (6, 3000, 40000, 512, 3, 700),          # rows long enough for several histogram passes; 159 parts
    (9, 2000, 9000, 256, 3, 1500),          # 36 base parts and 3 hyper parts
    (100, 150, 2100, 384, 3, 90),           # 65..128 rows: the weight-streaming kernel stores the base vocabulary's logits
    (150, 200, 3001, 256, 3, 200),          # 129..192 rows: the streaming kernel's widest build stores them
    (200, 120, 1800, 384, 3, 60),           # 193..256 rows: the tile kernel stores them, one row tile (rotated K walk)
    (700, 60, 2100, 128, 3, 40),            # three row tiles: base parts of two tiles (512 columns) each
    (1, 2000, 9000, 512, 3, 1500),          # one sequence: the dot-product units store the base vocabulary's logits
    (4, 600, 5000, 2560, 3, 300),           # four sequences
])
def test_truncated_draws_match_oracle_every_row(B, N, V, d, M, cap, whole_row_only):
    """Both ways of finding the kept prefix: the short list built from the parts with the largest maxima
    (settings with k up to 256 on rows with at least k parts, or a nucleus that closes early), and the passes
    over the whole row (everything else; all settings when whole_row_only)."""
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c3"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=3 * B + V)
    print(f"[case] truncated sampling B={B} V={V} d={d} cap={cap}", flush=True)
    lens = wl.make_lens(cfg)
    if B > 1:
        lens[1] = 0
    ctx, ref, E, H, w, d_E, d_W, d_H = _setup(cfg, lens)
    ctx.set_option(api.OPT_SAMPLE_KERNEL, whole_row_only)
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    lp = torch.empty(B, dtype=torch.float32, device="cuda")
    rows_logits = []
    for b in range(B):
        Wr = oracle.hyper_embed(E, cfg["dtype"], ref[b][1], cap, cfg["pool"], w)
        rows_logits.append(oracle.extended_logits(H[b:b + 1], E, Wr, len(ref[b][1]), cfg["dtype"])["logits"][0])
    settings = [(1.0, 1, 1.0), (0.7, 5, 1.0), (1.0, 50, 1.0), (1.0, 0, 0.3), (0.5, 0, 0.9), (1.3, 40, 0.8),
                (1.0, 10 ** 9, 0.9999), (2.0, 7000, 1.0), (0.05, 0, 0.5), (1.0, 2, 0.99), (0.9, 36, 1.0),
                (1.1, 39, 0.97), (1.0, 256, 1.0), (0.3, 257, 0.9)]
    n_decided = 0
    for si, (T, k, p) in enumerate(settings):
        seed, step = 900 + si, (si << 33) | 17
        ctx.extended_sample(d_H, 1, d_E, d_W, T, seed, step, tok, lp, top_k=k, top_p=p)
        torch.cuda.synchronize()
        tok_h, lp_h = tok.cpu().numpy(), lp.cpu().numpy()
        decided = sum(_check_truncated(rows_logits[b], T, k, p, seed, step, b, int(tok_h[b]), float(lp_h[b]))
                      for b in range(B))
        assert decided >= 0.8 * B - (1 if B < 8 else 0), (T, k, p, decided)
        n_decided += decided
    assert n_decided >= 0.8 * B * len(settings)
    ctx.close()


def test_truncation_with_equal_logits_is_decided_by_column():
    """H = 0 makes every logit equal: the order is the column order.  6000 columns exceed what one sort takes,
    so the cut is found by the by-column pass; 300 columns go through the sort."""
    import torch
    from paper_2506_01084_amd import api

    for V in (6000, 300):
        B, d, cap = 8, 128, 16
        ctx = api.Context(B=B, V=V, M=3, cap=cap, d=d, dtype="bf16")
        ctx.reset()
        g = torch.Generator(device="cuda")
        g.manual_seed(1)
        W = torch.randn((V, d), device="cuda", generator=g).to(torch.bfloat16)
        Wh = torch.zeros((B, cap, d), dtype=torch.bfloat16, device="cuda")
        H0 = torch.zeros((B, d), dtype=torch.bfloat16, device="cuda")
        tok = torch.empty(B, dtype=torch.int32, device="cuda")
        lp = torch.empty(B, dtype=torch.float32, device="cuda")
        for k, p, n_keep in ((5, 1.0, 5), (0, 0.5, V // 2), (4500, 0.9, min(4500, int(np.ceil(0.9 * V)))), (1, 0.2, 1)):
            seen = set()
            for step in range(6):
                ctx.extended_sample(H0, 1, W, Wh, 1.0, 77, step, tok, lp, top_k=k, top_p=p)
                torch.cuda.synchronize()
                t = tok.cpu().numpy()
                assert (t >= 0).all() and (t < n_keep + 1).all(), (V, k, p, t.max(), n_keep)   # +1: p * total in float
                assert np.allclose(lp.cpu().numpy(), -np.log(n_keep), atol=2e-2 + 1.0 / n_keep)
                seen.update(t.tolist())
                # the draw is the oracle's: all logits 0, the kept columns are 0 .. n_keep - 1
                for b in range(B):
                    _check_truncated(np.zeros(V), 1.0, k, p, 77, step, b, int(t[b]), float(lp[b]))
            assert len(seen) > 1 or n_keep == 1
        ctx.close()


def test_full_size_c3_truncated():
    import time
    import torch

    cfg = wl.CONFIGS["c3"]
    t0 = time.time()
    print("[case] full size truncated sampling step c3", flush=True)
    ctx, ref, E, H, w, d_E, d_W, d_H = _setup(cfg, np.full(cfg["B"], cfg["N"], dtype=np.int32))
    B = cfg["B"]
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    lp = torch.empty(B, dtype=torch.float32, device="cuda")
    W_host = storage_to_host(d_W, cfg["dtype"])
    lg = {}
    for b in (0, 40):
        lg[b] = oracle.extended_logits(H[b:b + 1], E, W_host[b], len(ref[b][1]), cfg["dtype"])["logits"][0]
    for T, k, p in ((0.8, 50, 0.9), (1.0, 0, 0.95), (1.0, 20000, 1.0)):
        seed, step = 4711, 99
        ctx.extended_sample(d_H, 1, d_E, d_W, T, seed, step, tok, lp, top_k=k, top_p=p)
        torch.cuda.synchronize()
        tok_h, lp_h = tok.cpu().numpy(), lp.cpu().numpy()
        for b in (0, 40):
            ok = _check_truncated(lg[b], T, k, p, seed, step, b, int(tok_h[b]), float(lp_h[b]))
            print(f"  T={T} k={k} p={p} seq {b}: token {tok_h[b]} logprob {lp_h[b]:.4f} decided {ok}  {time.time() - t0:.1f}s",
                  flush=True)
    ctx.close()


def test_many_sequences_picks_replay_in_a_graph():
    """Beyond 128 sequences the pick runs as tile kernel (base vocabulary) + hyper units + merge: the three picks
    (argmax, draw, filtered draw) captured once after an eager call, replayed three times with eager work in
    between, give the eager results every time (nothing is allocated or cleared by the host in between)."""
    import torch

    B, N, V, d, M, cap = 200, 120, 3001, 256, 3, 70
    cfg = wl.scaled(wl.CONFIGS["c3"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=77)
    print("[case] picks for 200 sequences, eager and graph", flush=True)
    ctx, ref, E, H, w, d_E, d_W, d_H = _setup(cfg, wl.make_lens(cfg))
    i32 = dict(dtype=torch.int32, device="cuda")
    f32 = dict(dtype=torch.float32, device="cuda")

    def bufs():
        return (torch.empty(B, **i32), torch.empty(B, **f32), torch.empty(B, **f32), torch.empty(B, **i32),
                torch.empty(B, **f32), torch.empty(B, **i32), torch.empty(B, **f32))

    def picks(o):
        ctx.extended_logits(d_H, 1, d_E, d_W, o[0], o[1], o[2], None)
        ctx.extended_sample(d_H, 1, d_E, d_W, 0.8, 11, 5, o[3], o[4])
        ctx.extended_sample(d_H, 1, d_E, d_W, 0.8, 11, 6, o[5], o[6], top_k=40, top_p=0.9)

    eager = bufs()
    picks(eager)
    torch.cuda.synchronize()
    out = bufs()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        picks(out)
    for rep in range(3):
        for t in out:
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for k in (0, 3, 5):
            assert torch.equal(out[k], eager[k]), f"replay {rep}: pick {k} differs from the eager call"
        for k in (1, 2, 4, 6):
            assert torch.equal(out[k], eager[k]), f"replay {rep}: value {k} differs from the eager call"
        assert np.isfinite(torch.randn(1 << 18, device="cuda").sum().item())        # eager work between replays
    ctx.close()


def test_filtered_draws_with_base_parts_of_two_tiles():
    """600 sequences over the full 128256-token vocabulary: three row tiles of the tile kernel, so its strips (the
    base parts the selection kernels' short list is built from) span two tiles = 512 columns.  Sampled rows
    against the oracle, every row valid."""
    import torch

    B, N, V, d, M, cap = 600, 40, 128256, 128, 3, 30
    cfg = wl.scaled(wl.CONFIGS["c3"], B=B, N=N, V=V, d=d, M=M, cap=cap, zipf_s=1.3, seed=5)
    print("[case] filtered sampling, 600 rows x 128256 columns", flush=True)
    ctx, ref, E, H, w, d_E, d_W, d_H = _setup(cfg, wl.make_lens(cfg))
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    lp = torch.empty(B, dtype=torch.float32, device="cuda")
    picks = [0, 1, 255, 256, 300, 511, 512, 599]
    rows_logits = {}
    for b in picks:
        Wr = oracle.hyper_embed(E, cfg["dtype"], ref[b][1], cap, cfg["pool"], w)
        rows_logits[b] = oracle.extended_logits(H[b:b + 1], E, Wr, len(ref[b][1]), cfg["dtype"])["logits"][0]
    for si, (T, k, p) in enumerate([(1.0, 50, 0.9), (0.7, 5, 1.0), (1.0, 0, 0.5), (1.2, 256, 0.95), (1.0, 1000, 1.0)]):
        seed, step = 40 + si, 7 * si
        ctx.extended_sample(d_H, 1, d_E, d_W, T, seed, step, tok, lp, top_k=k, top_p=p)
        torch.cuda.synchronize()
        tok_h, lp_h = tok.cpu().numpy(), lp.cpu().numpy()
        assert (tok_h >= 0).all() and all(tok_h[b] < V + len(ref[b][1]) for b in range(B))
        assert np.isfinite(lp_h).all() and (lp_h <= 1e-5).all()
        decided = sum(_check_truncated(rows_logits[b], T, k, p, seed, step, b, int(tok_h[b]), float(lp_h[b]))
                      for b in picks)
        assert decided >= len(picks) - 2, (T, k, p, decided)
    # the unfiltered draw at the same shape: the tile kernel's sampling epilogue with strips of two tiles
    for T, seed, step in ((1.0, 321, 0), (0.6, (9 << 32) | 4, 12)):
        ctx.extended_sample(d_H, 1, d_E, d_W, T, seed, step, tok, lp)
        torch.cuda.synchronize()
        tok_h, lp_h = tok.cpu().numpy(), lp.cpu().numpy()
        assert (tok_h >= 0).all() and all(tok_h[b] < V + len(ref[b][1]) for b in range(B))
        for b in picks:
            Wr = oracle.hyper_embed(E, cfg["dtype"], ref[b][1], cap, cfg["pool"], w)
            r = sampling.extended_sample(H[b:b + 1], E, Wr, len(ref[b][1]), cfg["dtype"], T, seed, step, row0=b)
            r["coords"] = [(seed, step, b)]
            _check_draws(r, tok_h[b:b + 1], lp_h[b:b + 1], T)
    ctx.close()
