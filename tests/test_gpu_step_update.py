"""GPU parity of z2z_step_update, the fused codebook side of a generation step (section 2.3, steps 9-10; the
hyper-embedding cache): it must leave exactly what an appended one-code z2z_lzw_decode followed by z2z_hyper_embed
of the newest entry leave -- codebook, statuses and cache rows bit for bit -- and both must agree with the oracle's
streaming decoder and pooling."""
import numpy as np
import pytest

import oracle
from paper_2506_01084_amd import workloads as wl

from helpers import gpu_encode, hyper_embed_bound, storage_to_host, torch_storage

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,B,V,d,M,cap,pool,history", [
    ("bf16", 6, 2000, 256, 3, 300, "mean", 400),
    ("bf16", 3, 500, 4096, 4, 64, "weighted", 90),      # widest row: eight waves share it
    ("f32", 5, 300, 100, 5, 40, "weighted", 30),         # 25 chunks: one wave, a ragged tail
    ("bf16", 4, 1000, 128, 3, 50, "mean", 0),           # no history: the codebooks start empty
    ("bf16", 2, 800, 64, 3, 0, "mean", 50),             # no codebook at all
])
def test_step_update_equals_the_two_calls_and_the_oracle(dtype, B, V, d, M, cap, pool, history):
    import torch
    from paper_2506_01084_amd import api

    cfg = dict(name="step", B=B, N=max(history, 1), V=V, d=d, dtype=dtype, M=M, cap=cap, zipf_s=1.2, copy_frac=0.4,
               span=(2, 6), mode="motif", pool=pool, seed=6100 + V + d)
    print(f"[case] step_update {dtype} B={B} V={V} d={d} M={M} cap={cap} {pool} history={history}", flush=True)
    w = wl.make_pool_weights(cfg)
    E = wl.make_embeddings(cfg)
    d_E = torch_storage(E, dtype)
    tokens = wl.make_tokens(cfg)
    streams = [oracle.LZWStream(V, M, cap) for _ in range(B)]
    ctxs, caches = [], []
    for _ in range(2):
        ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype=dtype, pool=pool, w=w.tolist())
        d_W = torch.full((B, cap, d), 1.0, dtype=ctx.torch_dtype, device="cuda")
        if history:
            gpu_encode(ctx, tokens, None)
        ctx.hyper_embed(d_E, d_W)
        ctxs.append(ctx)
        caches.append(d_W)
    if history:
        for b in range(B):
            streams[b].encode_chunk(tokens[b].tolist())
    rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 9))
    ones = torch.ones(B, dtype=torch.int32, device="cuda")
    n_steps = 40
    for t in range(n_steps):
        sizes = np.array([len(s.entries) for s in streams])
        codes = wl.make_step_codes(cfg, sizes, t)
        # every few steps: the one code that names the entry it creates, a code that names nothing, a repeat
        if t % 7 == 3:
            codes[0] = V + sizes[0]
        if t % 11 == 5:
            codes[B - 1] = V + sizes[B - 1] + 3
        if t % 5 == 4 and t > 0:
            codes[1 % B] = prev_codes[1 % B]
        prev_codes = codes.copy()
        stride = 1 + (t % 3)                                  # the code of sequence b sits at codes[b * stride]
        d_codes = torch.full((B, stride), -9, dtype=torch.int32, device="cuda")
        d_codes[:, 0] = torch.from_numpy(codes).cuda()
        outs = []
        for which, (ctx, d_W) in enumerate(zip(ctxs, caches)):
            n_tok = torch.full((B,), -7, dtype=torch.int32, device="cuda")
            st = torch.full((B,), -7, dtype=torch.int32, device="cuda")
            if which == 0:
                ctx.lzw_decode(d_codes, ones, None, n_tok, st, api.APPEND)
                ctx.hyper_embed(d_E, d_W, None, max_new=1)
            else:
                ctx.step_update(d_codes, d_E, d_W, n_tok, st)
            torch.cuda.synchronize()
            outs.append((n_tok.cpu().numpy(), st.cpu().numpy()))
        assert (outs[0][0] == outs[1][0]).all() and (outs[0][1] == outs[1][1]).all(), f"step {t}"
        for b in range(B):
            toks, rst = streams[b].decode_chunk([int(codes[b])])
            assert int(outs[1][1][b]) == rst, f"step {t} seq {b}: status {outs[1][1][b]} != {rst}"
            assert int(outs[1][0][b]) == len(toks)
        cb = [tuple(x.cpu().numpy() for x in ctx.codebook()) for ctx in ctxs]
        for x, y in zip(cb[0], cb[1]):
            assert (x == y).all(), f"step {t}: codebooks differ"
        assert cb[1][2].tolist() == [len(s.entries) for s in streams], f"step {t}: sizes differ from the oracle"
        assert torch.equal(caches[0], caches[1]), f"step {t}: cache rows differ"
    # the cache against the oracle's pooling of the final codebooks
    if cap:
        tol = 1e-5 if dtype == "f32" else 2e-2
        W_host = storage_to_host(caches[1], dtype)
        grew = 0
        for b in range(B):
            entries = streams[b].entries
            grew += len(entries)
            Wr = oracle.hyper_embed(E, dtype, entries, cap, pool, w)
            got, want = oracle.to_f64(W_host[b], dtype), oracle.to_f64(Wr, dtype)
            bound = hyper_embed_bound(E, dtype, entries, pool, w, cap)
            C = len(entries)
            assert (np.abs(got[:C] - want[:C]) <= tol * bound[:C] + 1e-30).all(), f"seq {b}"
        assert grew > 0
    for ctx in ctxs:
        ctx.close()
