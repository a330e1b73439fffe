"""GPU parity: lzw_encode / lzw_decode through the C ABI against the oracle, bit for bit."""
import numpy as np
import pytest

import oracle
from paper_2506_01084_amd import workloads as wl

from helpers import (assert_codebook_equal, gpu_decode, gpu_encode, oracle_encode_batch)

pytestmark = pytest.mark.gpu


def _ctx(cfg, **kw):
    from paper_2506_01084_amd import api

    args = dict(B=cfg.get("B"), V=cfg["V"], M=cfg["M"], cap=cfg["cap"], d=cfg.get("d", 64),
                dtype=cfg.get("dtype", "bf16"))
    args.update(kw)
    return api.Context(**args)


def _check_encode_decode(cfg, tokens, lens, lzw_kernel=0):
    from paper_2506_01084_amd import api

    B, N = tokens.shape
    V, M, cap = cfg["V"], cfg["M"], cfg["cap"]
    ctx = _ctx(cfg, B=B)
    ctx.set_option(api.OPT_LZW_KERNEL, lzw_kernel)
    ref = oracle_encode_batch(tokens, lens, V, M, cap)
    codes, n_codes, status = gpu_encode(ctx, tokens, lens)
    for b, (rc, rentries, rst) in enumerate(ref):
        assert int(status[b]) == rst, f"seq {b} status"
        assert int(n_codes[b]) == len(rc), f"seq {b}: {int(n_codes[b])} codes, oracle {len(rc)}"
        assert (codes[b, : len(rc)] == np.asarray(rc, dtype=np.int32)).all(), f"seq {b} codes differ"
    assert_codebook_equal(ctx, [r[1] for r in ref], M, cap)

    # decode the GPU's own codes in a fresh context: tokens and codebook must come back
    ctx2 = _ctx(cfg, B=B)
    ctx2.set_option(api.OPT_LZW_KERNEL, lzw_kernel)
    toks, n_tok, st = gpu_decode(ctx2, codes, n_codes, out_stride=max(N, 1))
    for b in range(B):
        L = int(lens[b])
        rt, _, rst = oracle.lzw_decode(ref[b][0], V, M, cap)
        assert int(st[b]) == rst == 0
        assert int(n_tok[b]) == len(rt) == L
        assert (toks[b, :L] == tokens[b, :L]).all(), f"seq {b} round trip"
    assert_codebook_equal(ctx2, [r[1] for r in ref], M, cap)
    ctx.close()
    ctx2.close()


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_full_size_configs_bit_exact(name):
    cfg = wl.CONFIGS[name]
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg)
    print(f"[case] lzw full size {name} B={cfg['B']} N={cfg['N']} M={cfg['M']} cap={cfg['cap']}", flush=True)
    _check_encode_decode(cfg, tokens, lens)


@pytest.mark.parametrize("name", ["c2", "c5"])
def test_global_table_variant_bit_exact(name):
    """The variant that keeps the hash table in global memory (used for huge capacities and short appends)."""
    cfg = wl.scaled(wl.CONFIGS[name], B=3, N=3000)
    tokens = wl.make_tokens(cfg)
    print(f"[case] lzw global-table variant {name}", flush=True)
    _check_encode_decode(cfg, tokens, wl.make_lens(cfg), lzw_kernel=2)


@pytest.mark.parametrize("name", ["c2", "c4", "c5"])
def test_one_wave_per_sequence_variant_bit_exact(name):
    """Few long sequences take the kernels with four waves per sequence by default; the one-wave kernels (what
    calls with many sequences run) on the same inputs."""
    cfg = wl.CONFIGS[name]
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg)
    print(f"[case] lzw one wave per sequence {name}", flush=True)
    _check_encode_decode(cfg, tokens, lens, lzw_kernel=4)


@pytest.mark.parametrize("name", ["c2", "c4"])
def test_serial_decoder_variant_bit_exact(name):
    """The one-code-at-a-time decoder (the one short appended calls take), forced on long streams."""
    cfg = wl.scaled(wl.CONFIGS[name], B=3, N=3000)
    tokens = wl.make_tokens(cfg)
    print(f"[case] lzw serial-decoder variant {name}", flush=True)
    _check_encode_decode(cfg, tokens, wl.make_lens(cfg), lzw_kernel=3)


def test_ragged_and_degenerate_lengths():
    cfg = wl.scaled(wl.CONFIGS["c1"], B=8, N=777)
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg, ragged=True)
    assert 0 in lens and 1 in lens and cfg["N"] in lens
    print("[case] lzw ragged lens", lens.tolist(), flush=True)
    _check_encode_decode(cfg, tokens, lens)


@pytest.mark.parametrize("V,M,cap", [(2, 3, 50), (3, 8, 200), (5, 1, 64), (4, 4, 0), (2, 5, 3), (1, 8, 16)])
def test_tiny_alphabets_and_limits(V, M, cap):
    """Small alphabets make repeats, the just-created-entry case and a full codebook frequent."""
    rng = np.random.default_rng(100 * V + 10 * M + cap)
    B, N = 6, 500
    tokens = rng.integers(0, V, size=(B, N)).astype(np.int32)
    tokens[0] = 0                                   # constant sequence
    lens = np.array([N, N, 63, 64, 65, 129], dtype=np.int32)
    print(f"[case] lzw tiny alphabet V={V} M={M} cap={cap}", flush=True)
    _check_encode_decode(dict(V=V, M=M, cap=cap), tokens, lens)


@pytest.mark.parametrize("B", [300, 1100])
def test_many_sequences_per_call(B):
    """Hundreds and thousands of sequences in one call: the library sizes its tables for occupancy (smaller
    LDS tables from 256 sequences, the table in global memory from 1024), results unchanged."""
    cfg = wl.scaled(wl.CONFIGS["c4"], B=B, N=300, V=500, cap=256, seed=B)
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg)
    print(f"[case] lzw many sequences B={B}", flush=True)
    _check_encode_decode(cfg, tokens, lens)


@pytest.mark.parametrize("B,N", [(200, 700), (700, 2100)])
def test_many_long_sequences_on_the_four_wave_kernels(B, N):
    """Hundreds of sequences of 512 tokens or more still take four waves each (several workgroups per CU, the
    smaller tables): ragged lengths across every window boundary, results unchanged."""
    cfg = wl.scaled(wl.CONFIGS["c4"], B=B, N=N, V=900, cap=700, seed=B + N)
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg, ragged=True)
    lens[:8] = [N, 0, 1, 255, 256, 257, 512, min(N, 1025)]
    print(f"[case] lzw four-wave kernels B={B} N={N}", flush=True)
    _check_encode_decode(cfg, tokens, lens)


@pytest.mark.parametrize("B,V,M,cap,N", [(700, 300, 3, 500, 2100), (1024, 70000, 8, 3000, 4097)])
def test_four_wave_kernels_with_many_workgroups_in_flight_are_deterministic(B, V, M, cap, N):
    """Hundreds of four-wave workgroups at once (table in LDS for 700 sequences, in global memory for 1024), on
    streams of short runs whose codebooks fill up early: the code of the round that names the entry being made
    is handled by all four waves together, and a wave that looked the edge up after wave 0 had stored it used
    to take the other branch.  Eight decodes of the same codes and three encodes must agree with the input and
    with one another."""
    from paper_2506_01084_amd import api

    rng = np.random.default_rng(B)
    tokens = np.ascontiguousarray(np.repeat(rng.integers(0, V, size=(B, N // 5 + 1)), 5, axis=1)[:, :N].astype(np.int32))
    lens = rng.integers(0, N + 1, size=B).astype(np.int32)
    lens[0] = N
    print(f"[case] lzw four-wave kernels, {B} workgroups in flight", flush=True)
    cfg = dict(V=V, M=M, cap=cap)
    ctx = _ctx(cfg, B=B)
    first = None
    for rep in range(3):
        codes, n_codes, status = gpu_encode(ctx, tokens, lens)
        assert (status == 0).all()
        if first is None:
            first = (codes.copy(), n_codes.copy())
        else:
            assert (n_codes == first[1]).all()
            assert all((codes[b, :n_codes[b]] == first[0][b, :n_codes[b]]).all() for b in range(B)), f"encode run {rep}"
    for b in rng.choice(B, size=16, replace=False):
        rc, _, rst = oracle.lzw_encode(tokens[b, :int(lens[b])].tolist(), V, M, cap)
        assert rst == 0 and int(n_codes[b]) == len(rc) and (codes[b, :len(rc)] == np.asarray(rc, dtype=np.int32)).all()
    for rep in range(8):
        ctx2 = _ctx(cfg, B=B)
        toks, n_tok, st = gpu_decode(ctx2, codes, n_codes, out_stride=N)
        bad = [b for b in range(B)
               if int(st[b]) != 0 or int(n_tok[b]) != int(lens[b]) or not (toks[b, :lens[b]] == tokens[b, :lens[b]]).all()]
        assert not bad, f"decode run {rep}: sequences {bad[:8]}"
        ctx2.close()
    ctx.close()


def test_largest_ids_capacity_and_merge_size():
    """The limits of the ID packing: V + cap = 2^24, cap = 65535, M = 8 (codes and tokens up to 2^24 - 1 in
    the hash slots, entry indices up to 65534, the table in global memory)."""
    cap, M = 65535, 8
    V = (1 << 24) - cap
    rng = np.random.default_rng(24)
    B, N = 2, 150000
    # a few hundred distinct IDs from the top and the bottom of the range, so that the codebook fills up
    alphabet = np.concatenate([np.arange(V - 200, V), np.arange(0, 200)]).astype(np.int64)
    tokens = alphabet[rng.integers(0, len(alphabet), size=(B, N))].astype(np.int32)
    tokens[1, : N // 3] = np.array([V - 1, 0, V - 2])[rng.integers(0, 3, size=N // 3)]   # three IDs: phrases reach M
    lens = np.array([N, N - 77], dtype=np.int32)
    print(f"[case] lzw limits V={V} M={M} cap={cap}", flush=True)
    ref = oracle_encode_batch(tokens, lens, V, M, cap)
    assert all(len(r[1]) == cap for r in ref), "the case must fill the codebooks"
    assert max(len(e) for e in ref[1][1]) == M, "the case must reach the merge limit"
    _check_encode_decode(dict(V=V, M=M, cap=cap, d=8), tokens, lens)


def test_bad_token_and_short_output():
    from paper_2506_01084_amd import api

    V, M, cap = 50, 3, 64
    rng = np.random.default_rng(5)
    B, N = 4, 300
    tokens = rng.integers(0, 6, size=(B, N)).astype(np.int32)
    tokens[1, 100] = V          # out of range
    tokens[2, 0] = -3           # out of range at the very start
    lens = np.full(B, N, dtype=np.int32)
    ctx = _ctx(dict(B=B, V=V, M=M, cap=cap))
    codes, n_codes, status = gpu_encode(ctx, tokens, lens)
    for b in range(B):
        rc, rentries, rst = oracle.lzw_encode(tokens[b].tolist(), V, M, cap)
        assert int(status[b]) == rst
        assert int(n_codes[b]) == len(rc) and (codes[b, : len(rc)] == np.asarray(rc, dtype=np.int32)).all()
    assert status.tolist() == [0, api.ST_BAD_TOKEN, api.ST_BAD_TOKEN, 0]
    # output row too short: the first out_stride codes are still the oracle's, status says overflow
    rc0, _, _ = oracle.lzw_encode(tokens[0].tolist(), V, M, cap)
    short = len(rc0) - 5
    codes, n_codes, status = gpu_encode(ctx, tokens, lens, out_stride=short)
    assert int(status[0]) & api.ST_OVERFLOW and int(n_codes[0]) == short
    assert (codes[0, :short] == np.asarray(rc0[:short], dtype=np.int32)).all()
    ctx.close()


@pytest.mark.parametrize("width", [8, 100])      # 8: the one-code-at-a-time kernel, 100: the round kernel
def test_decoder_error_paths(width):
    from paper_2506_01084_amd import api

    V, M, cap = 3, 3, 32
    B = 5
    streams = [
        [0, 3, 4, 1],           # valid; 3 and 4 each name the entry made in that very step (previous phrase + its first token)
        [0, 1, 9],              # 9 names nothing
        [4, 0],                 # a hyper code with no previous phrase
        [0, -2, 1],             # negative
        [2, 2, 2, 2],           # valid
    ]
    n = np.array([len(s) for s in streams], dtype=np.int32)
    codes = np.zeros((B, width), dtype=np.int32)
    for b, s in enumerate(streams):
        codes[b, : len(s)] = s
    ctx = _ctx(dict(B=B, V=V, M=M, cap=cap))
    toks, n_tok, st = gpu_decode(ctx, codes, n, out_stride=16)
    refs = [oracle.lzw_decode(s, V, M, cap) for s in streams]
    for b, (rt, rentries, rst) in enumerate(refs):
        assert int(st[b]) == rst, (b, int(st[b]), rst)
        assert int(n_tok[b]) == len(rt) and toks[b, : len(rt)].tolist() == rt
    assert [r[2] for r in refs] == [0, api.ST_BAD_CODE, api.ST_BAD_CODE, api.ST_BAD_CODE, 0]
    assert_codebook_equal(ctx, [r[1] for r in refs], M, cap)
    # short output buffer
    toks, n_tok, st = gpu_decode(ctx, codes, n, out_stride=3)
    for b, s in enumerate(streams):
        rt, _, rst = oracle.lzw_decode(s, V, M, cap, max_tokens=3)
        assert int(st[b]) == rst and int(n_tok[b]) == len(rt) and toks[b, : len(rt)].tolist() == rt
    ctx.close()


def _model_like_stream(rng, V, M, cap, n, p_fresh=0.05, p_entry=0.5):
    """Codes a model might emit: any base token or existing entry, now and then the not-yet-defined
    code; not what a greedy parse would produce (edges repeat, entries go unused)."""
    s = oracle.LZWStream(V, M, cap)
    codes = []
    for _ in range(n):
        C = len(s.entries)
        u = rng.random()
        if u < p_fresh and s.prev is not None:
            k = V + C                     # may or may not be acceptable: the oracle decides
        elif u < p_fresh + p_entry and C > 0:
            # recent entries more often than old ones: names entries made a few codes ago
            k = V + (C - 1 - int(rng.integers(0, min(C, 6))) if rng.random() < 0.5 else int(rng.integers(0, C)))
        else:
            k = int(rng.integers(0, V))
        _, st = s.decode_chunk([k])
        if st != 0:
            continue                      # keep the stream valid; error streams are built separately
        codes.append(k)
    return codes


@pytest.mark.parametrize("V,M,cap,lzw_kernel", [(3, 3, 40, 0), (6, 4, 300, 0), (50, 5, 2000, 0), (4, 2, 1000, 0),
                                                (6, 4, 300, 2), (2, 8, 500, 0), (6, 4, 300, 4), (50, 5, 2000, 4)])
def test_decoder_on_streams_no_greedy_parse_produces(V, M, cap, lzw_kernel):
    """Repeated edges inside a round, codes naming entries a few codes old, the not-yet-defined code,
    then a bad code in the middle and a short output row: all against the oracle's decoder."""
    from paper_2506_01084_amd import api

    rng = np.random.default_rng(1000 * V + M)
    B, n = 6, 700
    streams = [_model_like_stream(rng, V, M, cap, n - 37 * b) for b in range(B)]
    streams[4] = streams[4][:300] + [V + cap + 5] + streams[4][300:]          # names nothing
    streams[5] = streams[5][:129] + [-1] + streams[5][129:]
    width = max(len(s) for s in streams)
    codes = np.zeros((B, width), dtype=np.int32)
    for b, s in enumerate(streams):
        codes[b, : len(s)] = s
    n_codes = np.array([len(s) for s in streams], dtype=np.int32)
    print(f"[case] model-like streams V={V} M={M} cap={cap} kernel={lzw_kernel}", flush=True)
    for out_stride in (width * M, 333):
        ctx = _ctx(dict(B=B, V=V, M=M, cap=cap))
        ctx.set_option(api.OPT_LZW_KERNEL, lzw_kernel)
        toks, n_tok, st = gpu_decode(ctx, codes, n_codes, out_stride=out_stride)
        refs = [oracle.lzw_decode(s, V, M, cap, max_tokens=out_stride) for s in streams]
        for b, (rt, _, rst) in enumerate(refs):
            assert int(st[b]) == rst, (b, int(st[b]), rst)
            assert int(n_tok[b]) == len(rt), (b, int(n_tok[b]), len(rt))
            assert toks[b, : len(rt)].tolist() == rt, f"seq {b} tokens"
        assert_codebook_equal(ctx, [r[1] for r in refs], M, cap)
        ctx.close()
    assert refs[4][2] & api.ST_BAD_CODE or refs[4][2] & api.ST_OVERFLOW


def test_chunked_append_decode_matches_stream_oracle():
    """Append-mode decode in chunks of mixed sizes (both decoder kernels), with and without a token output."""
    from paper_2506_01084_amd import api

    V, M, cap = 7, 4, 400
    B = 3
    rng = np.random.default_rng(77)
    streams = [_model_like_stream(rng, V, M, cap, 900) for _ in range(B)]
    n = min(len(s) for s in streams)
    codes = np.array([s[:n] for s in streams], dtype=np.int32)
    ctx = _ctx(dict(B=B, V=V, M=M, cap=cap))
    ref = [oracle.LZWStream(V, M, cap) for _ in range(B)]
    pos, first = 0, True
    while pos < n:
        step = int(rng.choice([1, 5, 9, 63, 64, 200]))
        chunk = np.ascontiguousarray(codes[:, pos:pos + step])
        with_out = bool(rng.integers(0, 2))
        toks, n_tok, st = gpu_decode(ctx, chunk, None, out_stride=chunk.shape[1] * M if with_out else 0,
                                     flags=api.RESET if first else api.APPEND)
        for b in range(B):
            rt, rst = ref[b].decode_chunk(chunk[b].tolist())
            assert int(st[b]) == rst == 0
            assert int(n_tok[b]) == len(rt)
            if with_out:
                assert toks[b, : len(rt)].tolist() == rt
        assert_codebook_equal(ctx, [list(r.entries) for r in ref], M, cap)
        pos += step
        first = False
    ctx.close()


def test_chunked_append_encode_matches_stream_oracle():
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c4"], B=3, N=2000, cap=512)
    V, M, cap = cfg["V"], cfg["M"], cfg["cap"]
    tokens = wl.make_tokens(cfg)
    B, N = tokens.shape
    ctx = _ctx(cfg)
    streams = [oracle.LZWStream(V, M, cap) for _ in range(B)]
    rng = np.random.default_rng(9)
    pos, first = 0, True
    all_codes = [[] for _ in range(B)]
    while pos < N:
        step = int(rng.choice([1, 2, 7, 64, 65, 300]))
        chunk = tokens[:, pos:pos + step]
        codes, n_codes, status = gpu_encode(ctx, np.ascontiguousarray(chunk), None,
                                            flags=api.RESET if first else api.APPEND)
        for b in range(B):
            rc, rst = streams[b].encode_chunk(chunk[b].tolist())
            assert int(status[b]) == rst == 0
            assert codes[b, : int(n_codes[b])].tolist() == rc, (b, pos, step)
            all_codes[b] += rc
        assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
        pos += step
        first = False
    for b in range(B):      # the joined stream decodes to the input with the same codebook
        rt, rentries, rst = oracle.lzw_decode(all_codes[b], V, M, cap)
        assert rst == 0 and rt == tokens[b].tolist() and rentries == streams[b].entries
    ctx.close()


def test_decode_steps_grow_codebook_by_at_most_one():
    """The per-step update of generation: one new code per sequence, codebook-only decode (no token output)."""
    from paper_2506_01084_amd import api

    cfg = wl.scaled(wl.CONFIGS["c3"], B=6, N=4096)
    V, M, cap = cfg["V"], cfg["M"], cfg["cap"]
    tokens = wl.make_tokens(cfg)
    B = cfg["B"]
    ctx = _ctx(cfg)
    streams = [oracle.LZWStream(V, M, cap) for _ in range(B)]
    codes, n_codes, status = gpu_encode(ctx, tokens, None)
    for b in range(B):
        rc, _ = streams[b].encode_chunk(tokens[b].tolist())
        assert codes[b, : len(rc)].tolist() == rc
    grew = 0
    for step in range(256):
        sizes = np.array([len(s.entries) for s in streams])
        new = wl.make_step_codes(cfg, sizes, step)
        _, n_tok, st = gpu_decode(ctx, new.reshape(B, 1), None, out_stride=0, flags=api.APPEND)
        for b in range(B):
            rt, rst = streams[b].decode_chunk([int(new[b])])
            assert int(st[b]) == rst == 0 and int(n_tok[b]) == len(rt)
            assert 0 <= len(streams[b].entries) - sizes[b] <= 1
            grew += len(streams[b].entries) - sizes[b]
        if step % 32 == 31 or step < 3:
            assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
    assert grew > 0
    assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
    ctx.close()


def test_repeatable_across_runs_and_sequence_order():
    """No cross-sequence sharing: shuffling the batch permutes the outputs and nothing else."""
    cfg = wl.scaled(wl.CONFIGS["c2"], B=8, N=2048)
    tokens = wl.make_tokens(cfg)
    ctx = _ctx(cfg)
    c1, n1, _ = gpu_encode(ctx, tokens, None)
    c2, n2, _ = gpu_encode(ctx, tokens, None)
    assert (c1 == c2).all() and (n1 == n2).all()
    perm = np.random.default_rng(1).permutation(cfg["B"])
    c3, n3, _ = gpu_encode(ctx, np.ascontiguousarray(tokens[perm]), None)
    assert (n3 == n1[perm]).all()
    for i, b in enumerate(perm):
        assert (c3[i, : n3[i]] == c1[b, : n1[b]]).all()
    ctx.close()


@pytest.mark.parametrize("narrow_only", [0, 4])      # 0: four waves per sequence for long calls; 4: one wave always
def test_long_calls_errors_appends_and_repeats_both_encoders(narrow_only):
    """Calls of 512 tokens and more with few sequences take the encoder with four waves per sequence (rounds of
    256 positions); everything a round can meet, against the oracle, for both encoders: an out-of-range token in
    any of the four windows, an output row that ends in any window, long appended chunks, streams that repeat
    their proposals (runs, short periods: rounds cut at the first repeat), the merge limit M = 8, a codebook
    that fills in the middle of a round."""
    from paper_2506_01084_amd import api

    rng = np.random.default_rng(17)
    V, M, cap = 40, 4, 300
    B, N = 6, 1500
    tokens = rng.integers(0, 7, size=(B, N)).astype(np.int32)
    for b, at in enumerate((3, 70, 130, 200, 700, 1499)):         # windows 0..3 of the first round, later rounds
        tokens[b, at] = V + b
    lens = np.full(B, N, dtype=np.int32)
    ctx = _ctx(dict(B=B, V=V, M=M, cap=cap))
    ctx.set_option(api.OPT_LZW_KERNEL, narrow_only)
    codes, n_codes, status = gpu_encode(ctx, tokens, lens)
    ref = oracle_encode_batch(tokens, lens, V, M, cap)
    for b, (rc, rentries, rst) in enumerate(ref):
        assert int(status[b]) == rst == api.ST_BAD_TOKEN
        assert int(n_codes[b]) == len(rc) and codes[b, :len(rc)].tolist() == rc, f"bad token, seq {b}"
    assert_codebook_equal(ctx, [r[1] for r in ref], M, cap)
    # output rows that end after 1, 40, 100, 170, 230 and 600 codes
    tokens = rng.integers(0, 7, size=(B, N)).astype(np.int32)
    ref = oracle_encode_batch(tokens, lens, V, M, cap)
    for short in (1, 40, 100, 170, 230, 600):
        codes, n_codes, status = gpu_encode(ctx, tokens, lens, out_stride=short)
        for b in range(B):
            assert int(status[b]) & api.ST_OVERFLOW and int(n_codes[b]) == short
            assert codes[b, :short].tolist() == ref[b][0][:short], f"short output {short}, seq {b}"
    ctx.close()

    # repetitive streams, deep merges, a codebook that fills mid-round; long appended chunks
    for V, M, cap, kind in ((1, 8, 100, "constant"), (3, 8, 40, "period"), (5, 3, 25, "runs"), (200, 5, 4000, "zipf")):
        B, N = 4, 2600
        if kind == "constant":
            tokens = np.zeros((B, N), dtype=np.int32)
        elif kind == "period":
            tokens = np.tile(rng.integers(0, V, size=(B, 5)), (1, N // 5 + 1))[:, :N].astype(np.int32)
        elif kind == "runs":
            tokens = np.repeat(rng.integers(0, V, size=(B, N // 7 + 1)), 7, axis=1)[:, :N].astype(np.int32)
        else:
            tokens = np.minimum(rng.zipf(1.2, size=(B, N)) - 1, V - 1).astype(np.int32)
        tokens = np.ascontiguousarray(tokens)
        ctx = _ctx(dict(B=B, V=V, M=M, cap=cap))
        ctx.set_option(api.OPT_LZW_KERNEL, narrow_only)
        streams = [oracle.LZWStream(V, M, cap) for _ in range(B)]
        pos, first = 0, True
        for step in (700, 513, 1, 900, 486):
            chunk = np.ascontiguousarray(tokens[:, pos:pos + step])
            lens = rng.integers(0, step + 1, size=B).astype(np.int32)
            lens[0] = step
            codes, n_codes, status = gpu_encode(ctx, chunk, lens, flags=api.RESET if first else api.APPEND)
            for b in range(B):
                rc, rst = streams[b].encode_chunk(chunk[b, :lens[b]].tolist())
                assert int(status[b]) == rst == 0
                assert codes[b, :int(n_codes[b])].tolist() == rc, (kind, b, pos, step)
            assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
            pos += step
            first = False
        ctx.close()


def test_short_appended_calls_in_wide_rows():
    """A call whose rows are long (so the launch picks the four-wave kernels) but whose sequences hold only a
    few elements this time: the length is known on the device only, and the kernel takes the short path."""
    from paper_2506_01084_amd import api

    V, M, cap = 30, 4, 500
    B, N = 5, 900
    rng = np.random.default_rng(23)
    tokens = rng.integers(0, 6, size=(B, N)).astype(np.int32)
    ctx = _ctx(dict(B=B, V=V, M=M, cap=cap))
    streams = [oracle.LZWStream(V, M, cap) for _ in range(B)]
    full = np.full(B, N, dtype=np.int32)
    codes, n_codes, st = gpu_encode(ctx, tokens, full)                       # a long call: four waves
    for b in range(B):
        assert codes[b, :n_codes[b]].tolist() == streams[b].encode_chunk(tokens[b].tolist())[0]
    for rep in range(4):                                                     # short ones in rows of 900
        more = rng.integers(0, 6, size=(B, N)).astype(np.int32)
        lens = rng.integers(0, 8, size=B).astype(np.int32)
        lens[0] = 64
        codes, n_codes, st = gpu_encode(ctx, more, lens, flags=api.APPEND)
        for b in range(B):
            rc, rst = streams[b].encode_chunk(more[b, :lens[b]].tolist())
            assert int(st[b]) == rst == 0 and codes[b, :n_codes[b]].tolist() == rc, (rep, b)
        assert_codebook_equal(ctx, [s.entries for s in streams], M, cap)
    # the same for the decoder: a second context follows the first one's code streams
    ctx2 = _ctx(dict(B=B, V=V, M=M, cap=cap))
    dec = [oracle.LZWStream(V, M, cap) for _ in range(B)]
    codes, n_codes, st = gpu_encode(ctx, tokens, full)                       # fresh long stream (RESET)
    toks, n_tok, st = gpu_decode(ctx2, codes, n_codes, out_stride=N)
    for b in range(B):
        rt, rst = dec[b].decode_chunk(codes[b, :n_codes[b]].tolist())
        assert int(st[b]) == rst == 0 and toks[b, :n_tok[b]].tolist() == rt == tokens[b].tolist()
    for rep in range(4):
        wide_rows = np.zeros((B, N), dtype=np.int32)
        cnt = rng.integers(0, 5, size=B).astype(np.int32)
        for b in range(B):
            C = len(dec[b].entries)
            for i in range(cnt[b]):
                wide_rows[b, i] = int(rng.integers(0, V + C))
        toks, n_tok, st = gpu_decode(ctx2, wide_rows, cnt, out_stride=64, flags=api.APPEND)
        for b in range(B):
            rt, rst = dec[b].decode_chunk(wide_rows[b, :cnt[b]].tolist())
            assert int(st[b]) == rst and toks[b, :n_tok[b]].tolist() == rt, (rep, b)
        assert_codebook_equal(ctx2, [s.entries for s in dec], M, cap)
    ctx.close()
    ctx2.close()
