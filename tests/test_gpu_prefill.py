"""GPU parity: codebook prefilling (the paper's discussion, "Codebook Management Strategy", item 2) through the
C ABI against the oracle: the entries and statuses after the prefill, and the codes, tokens and codebooks of a
parse / round trip that continues from it -- bit exact."""
import numpy as np
import pytest

import oracle
from oracle import LZWStream
from paper_2506_01084_amd import workloads as wl

from helpers import assert_codebook_equal, gpu_decode, gpu_encode

pytestmark = pytest.mark.gpu


def _pack(phrase_lists, n_max, M):
    B = len(phrase_lists)
    ph = np.full((B, n_max, M), -1, dtype=np.int32)
    ln = np.zeros((B, n_max), dtype=np.int32)
    cnt = np.zeros(B, dtype=np.int32)
    for b, lst in enumerate(phrase_lists):
        cnt[b] = len(lst)
        for i, p in enumerate(lst):
            ph[b, i, :min(len(p), M)] = p[:M]
            ln[b, i] = len(p)
    return ph, ln, cnt


def _prefill(ctx, phrase_lists, n_max, M, flags):
    import torch

    ph, ln, cnt = _pack(phrase_lists, n_max, M)
    B = len(phrase_lists)
    added = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    status = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ctx.codebook_prefill(torch.from_numpy(ph).cuda(), torch.from_numpy(ln).cuda(), torch.from_numpy(cnt).cuda(), added,
                         status, flags)
    torch.cuda.synchronize()
    return added.cpu().numpy(), status.cpu().numpy()


@pytest.mark.parametrize("B,N,V,M,cap", [(6, 400, 50, 3, 300), (3, 900, 2000, 4, 128), (260, 200, 30, 3, 64)])
def test_prefill_then_encode_and_decode_match_oracle(B, N, V, M, cap):
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, M=M, cap=cap, d=64, zipf_s=1.2, seed=B + V)
    print(f"[case] prefill B={B} N={N} V={V} M={M} cap={cap}", flush=True)
    tokens = wl.make_tokens(cfg)
    warm = wl.make_tokens(wl.scaled(cfg, seed=cfg["seed"] + 50))
    rng = np.random.default_rng(3)
    seeds = []
    for b in range(B):
        ent = oracle.lzw_encode(warm[b].tolist(), V, M, cap)[1]
        seeds.append([tuple(e) for e in ent[: int(rng.integers(0, min(len(ent), cap) + 1))]])
    seeds[0] = []                                          # one sequence without any
    n_max = max(len(s) for s in seeds) + 1
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=64, dtype="bf16")
    added, status = _prefill(ctx, seeds, n_max, M, api.RESET)
    streams = [LZWStream(V, M, cap) for _ in range(B)]
    for b in range(B):
        a, st = streams[b].prefill(seeds[b])
        assert (added[b], status[b]) == (a, st)
    assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
    # the parse continues from the prefilled codebooks
    lens = wl.make_lens(cfg, ragged=True)
    codes, n_codes, st = gpu_encode(ctx, tokens, lens, flags=api.APPEND)
    ref_codes = []
    for b in range(B):
        c, s = streams[b].encode_chunk(tokens[b, :lens[b]].tolist())
        ref_codes.append(c)
        assert st[b] == s and codes[b, :n_codes[b]].tolist() == c, f"seq {b}"
    assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
    # and back: a decoder that prefilled alike
    added2, status2 = _prefill(ctx, seeds, n_max, M, api.RESET)
    assert (added2 == added).all() and (status2 == status).all()
    toks, n_tok, st = gpu_decode(ctx, codes, n_codes, out_stride=N, flags=api.APPEND)
    for b in range(B):
        assert st[b] == 0 and n_tok[b] == lens[b] and (toks[b, :lens[b]] == tokens[b, :lens[b]]).all(), f"seq {b}"
    assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
    ctx.close()


def test_prefill_statuses_and_append():
    from paper_2506_01084_amd import api

    V, M, cap = 9, 3, 4
    lists = [
        [(1, 2), (1, 2, 3)],                               # fine
        [(1, 2, 3)],                                       # prefix unknown
        [(1, 2), (1, 2)],                                  # duplicate
        [(1,)],                                            # too short
        [(1, 2), (1, 2, 3), (1, 2, 3, 4)],                 # longer than M
        [(1, 9)],                                          # token out of range
        [(0, 1), (0, 2), (0, 3), (0, 4), (1, 1)],          # more than cap
        [],
    ]
    B = len(lists)
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=64, dtype="bf16")
    added, status = _prefill(ctx, lists, 6, 4 if False else M, api.RESET)
    streams = [LZWStream(V, M, cap) for _ in range(B)]
    for b in range(B):
        a, st = streams[b].prefill(lists[b])
        assert (added[b], status[b]) == (a, st), (b, added[b], status[b], a, st)
    assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
    # a second prefill in append mode adds to what is there
    more = [[(2, 2)] for _ in range(B)]
    added, status = _prefill(ctx, more, 1, M, api.APPEND)
    for b in range(B):
        a, st = streams[b].prefill(more[b])
        assert (added[b], status[b]) == (a, st), b
    assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
    ctx.close()


@pytest.mark.parametrize("B,N,V,M,cap", [(5, 500, 40, 3, 200), (3, 1200, 300, 5, 150), (130, 150, 20, 4, 64)])
def test_usage_and_prune_match_oracle_and_the_parse_goes_on(B, N, V, M, cap):
    import torch
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, N=N, V=V, M=M, cap=cap, d=64, zipf_s=1.1, seed=3 * B + V)
    print(f"[case] prune B={B} N={N} V={V} M={M} cap={cap}", flush=True)
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg, ragged=True)
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=64, dtype="bf16")
    codes, n_codes, st = gpu_encode(ctx, tokens, lens)
    streams = [LZWStream(V, M, cap) for _ in range(B)]
    ref_codes = [streams[b].encode_chunk(tokens[b, :lens[b]].tolist())[0] for b in range(B)]
    # usage
    usage = torch.zeros((B, cap), dtype=torch.int32, device="cuda")
    ctx.codebook_usage(torch.from_numpy(codes).cuda(), torch.from_numpy(n_codes).cuda(), usage)
    torch.cuda.synchronize()
    use_h = usage.cpu().numpy()
    rng = np.random.default_rng(5)
    keep = np.zeros((B, cap), dtype=np.int32)
    for b in range(B):
        want = streams[b].usage(ref_codes[b])
        assert use_h[b, :len(want)].tolist() == want and (use_h[b, len(want):] == 0).all(), f"usage seq {b}"
        # retention policy of the test: entries that were used, plus a random few
        keep[b, :len(want)] = (np.array(want) > 0) | (rng.random(len(want)) < 0.2) if want else 0
    keep[0] = 1                                            # one sequence keeps everything
    if B > 1:
        keep[1] = 0                                        # one keeps nothing
    # prune
    new_id = torch.full((B, cap), -9, dtype=torch.int32, device="cuda")
    n_kept = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    ctx.codebook_prune(torch.from_numpy(keep).cuda(), new_id, n_kept)
    torch.cuda.synchronize()
    nid_h, nk_h = new_id.cpu().numpy(), n_kept.cpu().numpy()
    for b in range(B):
        C_old = len(streams[b].entries)
        want_map = streams[b].prune(keep[b, :C_old].tolist())
        assert nid_h[b, :C_old].tolist() == want_map and (nid_h[b, C_old:] == -9).all(), f"map seq {b}"
        assert nk_h[b] == len(streams[b].entries)
    assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
    # the parse goes on from the pruned codebooks, and a decoder that holds the same codebooks follows it
    more = wl.make_tokens(wl.scaled(cfg, seed=cfg["seed"] + 1))
    codes2, n2, st2 = gpu_encode(ctx, more, lens, flags=api.APPEND)
    kept_entries = [list(s.entries) for s in streams]
    for b in range(B):
        c, s_ = streams[b].encode_chunk(more[b, :lens[b]].tolist())
        assert st2[b] == s_ and codes2[b, :n2[b]].tolist() == c, f"parse after prune, seq {b}"
    assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
    from test_gpu_prefill import _prefill as prefill    # the decoder side: prefill the survivors, then decode
    n_max = max(len(k) for k in kept_entries) + 1
    added, status = prefill(ctx, kept_entries, n_max, M, api.RESET)
    assert (status == 0).all()
    toks, n_tok, st3 = gpu_decode(ctx, codes2, n2, out_stride=N, flags=api.APPEND)
    for b in range(B):
        assert st3[b] == 0 and n_tok[b] == lens[b] and (toks[b, :lens[b]] == more[b, :lens[b]]).all(), f"round trip seq {b}"
    ctx.close()
