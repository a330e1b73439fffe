"""GPU test of z2z_extended_logits_static, the entry point for callers that cannot allocate device memory: its
partial reductions live in a static device array of the library instead of the context's growable buffer.

It shares z2z_extended_logits' kernels, so its outputs must be bit-identical to that entry point's (and with
them within the logits bars of the oracle).  Two calls in a row, the second smaller, share the array: what the
first left behind must not reach the second.  A call beyond the array's size is refused.  A call on a context
that has never sized its own buffers is captured into a HIP graph and replayed (an allocation there would break
the capture).
"""
import numpy as np
import pytest

import oracle
from paper_2506_01084_amd import workloads as wl

from helpers import check_logits_rows, gpu_encode, oracle_encode_batch, torch_storage

pytestmark = pytest.mark.gpu


def _setup(B, rows_per_seq, V, d, cap, seed, N=700):
    import torch
    from paper_2506_01084_amd import api

    cfg = dict(name="noalloc", B=B, N=N, V=V, d=d, dtype="bf16", M=3, cap=cap, zipf_s=1.2, copy_frac=0.4, span=(2, 6),
               mode="motif", pool="mean", seed=seed)
    tokens = wl.make_tokens(cfg)
    lens = wl.make_lens(cfg)
    if B > 2:
        lens[1] = 0
    E = wl.make_embeddings(cfg)
    H = wl.make_hidden(cfg, B * rows_per_seq)
    ctx = api.Context(B=B, V=V, M=3, cap=cap, d=d, dtype="bf16", pool="mean")
    gpu_encode(ctx, tokens, lens)
    ref = oracle_encode_batch(tokens, lens, V, 3, cap)
    d_E = torch_storage(E, "bf16")
    d_W = torch.zeros((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.hyper_embed(d_E, d_W)
    d_H = torch_storage(H, "bf16")
    torch.cuda.synchronize()
    return cfg, ctx, ref, E, H, d_E, d_W, d_H


def _outputs(rows):
    import torch

    return (torch.full((rows,), -3, dtype=torch.int32, device="cuda"),
            torch.full((rows,), 55.0, dtype=torch.float32, device="cuda"),
            torch.full((rows,), 55.0, dtype=torch.float32, device="cuda"))


def _check_against_oracle(cfg, ref, E, H, rows_per_seq, outs):
    am, mx, lse = (t.cpu().numpy() for t in outs)
    for b in range(cfg["B"]):
        Wr = oracle.hyper_embed(E, "bf16", ref[b][1], cfg["cap"], "mean", None)
        sl = slice(b * rows_per_seq, (b + 1) * rows_per_seq)
        r = oracle.extended_logits(H[sl], E, Wr, len(ref[b][1]), "bf16")
        check_logits_rows(r, am[sl], mx[sl], lse[sl], None)


def test_static_entry_point_matches_the_allocating_one_twice_in_a_row_and_captures():
    import torch
    from paper_2506_01084_amd import api

    # ---- first call: a prefill shape (tile kernels), on a context whose own buffers were never sized -------
    print("[case] static entry point, prefill shape then a smaller decode shape", flush=True)
    cfg1, ctx1, ref1, E1, H1, d_E1, d_W1, d_H1 = _setup(B=5, rows_per_seq=300, V=3000, d=128, cap=400, seed=8101)
    cfg2, ctx2, ref2, E2, H2, d_E2, d_W2, d_H2 = _setup(B=3, rows_per_seq=1, V=900, d=256, cap=200, seed=8102)
    st1, st2 = _outputs(5 * 300), _outputs(3)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    ctx1.extended_logits_static(d_H1, 300, d_E1, d_W1, *st1)
    # ---- second call, smaller, other context and shape (one row per sequence: the decode kernel) ----------
    ctx2.extended_logits_static(d_H2, 1, d_E2, d_W2, *st2)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "the static entry point changed the free device memory"
    # ---- the allocating entry point on the same inputs: bit-identical -------------------------------------
    for ctx, d_H, rps, d_E, d_W, st, cfg, ref, E, H in ((ctx1, d_H1, 300, d_E1, d_W1, st1, cfg1, ref1, E1, H1),
                                                       (ctx2, d_H2, 1, d_E2, d_W2, st2, cfg2, ref2, E2, H2)):
        dyn = _outputs(d_H.shape[0])
        ctx.extended_logits(d_H, rps, d_E, d_W, *dyn)
        torch.cuda.synchronize()
        for a, b in zip(st, dyn):
            assert torch.equal(a, b), "static and allocating entry points disagree"
        _check_against_oracle(cfg, ref, E, H, rps, st)
    # ---- and the first shape again after the smaller one -------------------------------------------------
    again = _outputs(5 * 300)
    ctx1.extended_logits_static(d_H1, 300, d_E1, d_W1, *again)
    torch.cuda.synchronize()
    for a, b in zip(st1, again):
        assert torch.equal(a, b)
    # ---- with the full-logits output (general tile kernel) ------------------------------------------------
    full_s = torch.zeros((3, 900 + 200), dtype=torch.float32, device="cuda")
    full_d = torch.ones((3, 900 + 200), dtype=torch.float32, device="cuda")
    o_s, o_d = _outputs(3), _outputs(3)
    ctx2.extended_logits_static(d_H2, 1, d_E2, d_W2, *o_s, full_s)
    ctx2.extended_logits(d_H2, 1, d_E2, d_W2, *o_d, full_d)
    torch.cuda.synchronize()
    assert torch.equal(full_s, full_d) and all(torch.equal(a, b) for a, b in zip(o_s, o_d))
    ctx1.close()
    ctx2.close()


def test_static_entry_point_refuses_what_does_not_fit():
    import torch
    from paper_2506_01084_amd import api

    V, d, rows = 128256, 64, 40000         # 126 strips of the base vocabulary x 40000 rows > 2^22 elements
    ctx = api.Context(B=1, V=V, M=3, cap=0, d=d, dtype="bf16", pool="mean")
    d_W = torch.zeros((V, d), dtype=torch.bfloat16, device="cuda")
    d_Wh = torch.zeros((1, 0, d), dtype=torch.bfloat16, device="cuda")
    d_H = torch.zeros((rows, d), dtype=torch.bfloat16, device="cuda")
    outs = _outputs(rows)
    with pytest.raises(api.Z2ZError) as e:
        ctx.extended_logits_static(d_H, rows, d_W, d_Wh, *outs)
    assert e.value.code == api.E_LIMIT
    torch.cuda.synchronize()
    assert (outs[0] == -3).all() and (outs[1] == 55.0).all()       # nothing was enqueued
    # just inside the limit: 126 * 33288 <= 2^22
    rows_ok = api.STATIC_PARTS // 126
    d_H2 = torch.zeros((rows_ok, d), dtype=torch.bfloat16, device="cuda")
    outs2 = _outputs(rows_ok)
    ctx.extended_logits_static(d_H2, rows_ok, d_W, d_Wh, *outs2)
    torch.cuda.synchronize()
    assert (outs2[0] == 0).all() and (outs2[1] == 0).all()         # H = 0: every logit 0, lowest column wins
    assert np.allclose(outs2[2].cpu().numpy(), np.log(V), atol=1e-4)
    ctx.close()


def test_static_entry_point_under_graph_capture_on_a_fresh_context():
    """A fresh context has no buffer of its own for the partials; the allocating entry point would have to call
    hipMalloc inside the capture.  The static one captures and every replay reproduces the eager result."""
    import torch
    from paper_2506_01084_amd import api

    cfg, ctx, ref, E, H, d_E, d_W, d_H = _setup(B=4, rows_per_seq=1, V=2000, d=256, cap=300, seed=8103)
    outs = _outputs(4)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    refused = None
    with torch.cuda.graph(graph, stream=side):
        # the allocating entry point would have to size the context's buffer now: it says so and enqueues
        # nothing, and the capture goes on
        try:
            ctx.extended_logits(d_H, 1, d_E, d_W, *_outputs(4))
        except api.Z2ZError as e:
            refused = e.code
        ctx.extended_logits_static(d_H, 1, d_E, d_W, *outs)
    assert refused == api.E_CAPTURE
    eager = _outputs(4)
    ctx.extended_logits_static(d_H, 1, d_E, d_W, *eager)
    torch.cuda.synchronize()
    _check_against_oracle(cfg, ref, E, H, 1, eager)
    for rep in range(3):
        for t in outs:
            t.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(outs, eager):
            assert torch.equal(a, b), f"replay {rep} differs from the eager call"
        junk = torch.randn(1 << 18, device="cuda").sum().item()      # unrelated eager work between replays
        assert np.isfinite(junk)
    ctx.close()
