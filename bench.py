"""Benchmark of the zip2zip dynamic-vocabulary hot path on one MI355X.

One "step" is one pass of the whole path over one batch of configuration 2 (prefill at Llama-3-8B
shapes: 8 x 4096 tokens, V = 128256, d = 4096 bf16, M = 3, cap = 2048), inputs resident in HBM:

    lzw_encode (all tokens)  ->  hyper_embed (all entries)  ->  extended_logits (all 32768 rows)
    ->  one generation step on the same batch: lzw_decode append of one new code per sequence (the
        argmax of its last position), hyper_embed of the new entry, extended_logits for 8 rows
    ->  lzw_decode of the whole code stream back to base tokens

`value` is base tokens per second of that whole step.  The decode step of configuration 3 (64 sequences
with 8192-token histories, HBM-bound) is timed separately in the same run and reported in `decode_step`.
The learned hyper-encoder (a two-layer transformer over every entry's slots, in place of the averaging one) is
timed on configuration 2's codebooks and reported in `hyper_encode`; the training-side loss over the extended
vocabulary and its gradient, on configuration 2, in `nll_backward`.
The CPU oracle is timed on a bounded sample of the same workload as `cpu_baseline`.

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E

# HBM-side bytes per launch (fetch + write) from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs whose
# summaries are committed under profiles/ (counter values scaled by a 1 GiB copy of known traffic).
# They are measurements of these exact workloads, not computed here: a different workload reports null.
TRAFFIC_BYTES = {
    "logits_fast_kernel<0>@c2": 53.88e9 + 0.070e9,
    "logits_decode_kernel@c3": 3.211e9 + 0.003e9,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def to_device_bf16(torch, bits, dtype="bf16"):
    """Host uint16 bf16 bit patterns -> device bfloat16 tensor (memory plumbing only)."""
    import numpy as np

    assert dtype == "bf16"
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


class Stage:
    """Accumulates the time between two torch events recorded on the current stream."""

    def __init__(self, torch, n):
        self.torch = torch
        self.ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        self.i = 0

    def __enter__(self):
        self.ev[self.i][0].record()

    def __exit__(self, *exc):
        self.ev[self.i][1].record()
        self.i += 1

    def total_ms(self):
        return sum(a.elapsed_time(b) for a, b in self.ev[: self.i])


def run_prefill_workload(args, torch, api, wl):
    cfg = wl.CONFIGS["c2"]
    B, N, V, M, cap, d = (cfg[k] for k in ("B", "N", "V", "M", "cap", "d"))
    rows = B * N
    t0 = time.time()
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    H = wl.make_hidden(cfg, rows)
    log(f"[bench] c2 inputs generated in {time.time() - t0:.1f}s")
    d_tok = torch.from_numpy(tokens).cuda()
    d_E = to_device_bf16(torch, E, "bf16")          # tied: the matrix pooled is the LM head
    d_H = to_device_bf16(torch, H, "bf16")
    d_Hdec = d_H[N - 1::N].contiguous()             # one hidden row per sequence for the generation step
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype="bf16", pool="mean")
    i32 = dict(dtype=torch.int32, device="cuda")
    d_codes = torch.empty((B, N), **i32)
    d_ncodes = torch.empty(B, **i32)
    d_status = torch.empty(B, **i32)
    d_W = torch.empty((B, cap, d), dtype=torch.bfloat16, device="cuda")
    d_am = torch.empty(rows, **i32)
    d_mx = torch.empty(rows, dtype=torch.float32, device="cuda")
    d_lse = torch.empty(rows, dtype=torch.float32, device="cuda")
    d_one = torch.ones(B, **i32)
    d_ntok1 = torch.empty(B, **i32)
    d_st1 = torch.empty(B, **i32)
    d_am1 = torch.empty(B, **i32)
    d_mx1 = torch.empty(B, dtype=torch.float32, device="cuda")
    d_lse1 = torch.empty(B, dtype=torch.float32, device="cuda")
    d_back = torch.empty((B, N), **i32)
    d_nback = torch.empty(B, **i32)
    d_st2 = torch.empty(B, **i32)
    size_view = ctx.codebook()[2]

    names = ["lzw_encode", "hyper_embed", "extended_logits", "generation_step", "lzw_decode"]
    stages = None

    def step():
        with stages["lzw_encode"]:
            ctx.lzw_encode(d_tok, None, d_codes, d_ncodes, d_status, api.RESET)
        with stages["hyper_embed"]:
            ctx.hyper_embed(d_E, d_W)
        with stages["extended_logits"]:
            # the library brackets this call's dominant kernel (the base-vocabulary tile kernel) with HIP
            # events on this stream; the switch is host-side only and does not synchronise
            ctx.set_option(api.OPT_TIMING, 1)
            ctx.extended_logits(d_H, N, d_E, d_W, d_am, d_mx, d_lse, None)
            ctx.set_option(api.OPT_TIMING, 0)
        with stages["generation_step"]:
            # code of sequence b = argmax of its last position = element b*N of the view starting at N-1
            ctx.lzw_decode(d_am[N - 1:], d_one, None, d_ntok1, d_st1, api.APPEND, stride=N)
            ctx.hyper_embed(d_E, d_W, None, max_new=1)
            ctx.extended_logits(d_Hdec, 1, d_E, d_W, d_am1, d_mx1, d_lse1, None)
        with stages["lzw_decode"]:
            ctx.lzw_decode(d_codes, d_ncodes, d_back, d_nback, d_st2, api.RESET)

    stages = {n: Stage(torch, args.warmup) for n in names}
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.read_timing()
    stages = {n: Stage(torch, args.steps) for n in names}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_ms, launches = ctx.read_timing()

    # sanity inside the bench: statuses clean, round trip exact
    assert int(d_status.abs().sum()) == 0 and int(d_st1.abs().sum()) == 0 and int(d_st2.abs().sum()) == 0
    assert torch.equal(d_back, d_tok), "lzw_decode(lzw_encode(x)) != x"
    sizes = size_view.cpu().numpy()
    ncodes = d_ncodes.cpu().numpy()
    # how many of the entries the code stream ever names (the paper's discussion: about a quarter on its data)
    d_usage = torch.zeros((B, cap), **i32)
    ctx.codebook_usage(d_codes, d_ncodes, d_usage)
    reused = float((d_usage > 0).sum().item()) / max(1.0, float(sizes.sum()))

    ms_per_step = dt * 1e3 / args.steps
    stage_ms = {n: stages[n].total_ms() / args.steps for n in names}
    flops_base = 2.0 * rows * d * V
    flops_all = 2.0 * rows * d * (V + float(sizes.mean()))
    out = dict(ms_per_step=ms_per_step, stage_ms=stage_ms, kernel_ms_total=kernel_ms, kernel_launches=launches,
               flops_base=flops_base, flops_all=flops_all, sizes=sizes.tolist(), n_codes=ncodes.tolist(),
               tokens=B * N, cfg=cfg, entries_reused_frac=reused)
    host = dict(tokens=tokens, E=E, H=H)
    ctx.close()
    return out, host


def run_decode_workload(args, torch, api, wl):
    """Configuration 3: one decode step = codebook update for one new code per sequence, hyper_embed of
    the new entry, extended_logits for one hidden row per sequence."""
    cfg = wl.CONFIGS["c3"]
    B, N, V, M, cap, d = (cfg[k] for k in ("B", "N", "V", "M", "cap", "d"))
    t0 = time.time()
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    H = wl.make_hidden(cfg, B)
    log(f"[bench] c3 inputs generated in {time.time() - t0:.1f}s")
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype="bf16", pool="mean")
    i32 = dict(dtype=torch.int32, device="cuda")
    d_tok = torch.from_numpy(tokens).cuda()
    d_codes = torch.empty((B, N), **i32)
    d_n = torch.empty(B, **i32)
    d_st = torch.empty(B, **i32)
    d_E = to_device_bf16(torch, E, "bf16")
    d_H = to_device_bf16(torch, H, "bf16")
    d_W = torch.empty((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.lzw_encode(d_tok, None, d_codes, d_n, d_st, api.RESET)     # history (untimed)
    ctx.hyper_embed(d_E, d_W)
    torch.cuda.synchronize()
    size_view = ctx.codebook()[2]
    sizes = size_view.cpu().numpy()
    timed = max(args.steps, 50)          # a step is ~0.6 ms: enough of them that the pipeline fill does not show
    n_steps = args.warmup + timed
    new_codes = [torch.from_numpy(wl.make_step_codes(cfg, sizes, s).reshape(B, 1)).cuda() for s in range(n_steps)]
    d_ntok = torch.empty(B, **i32)
    d_am = torch.empty(B, **i32)
    d_mx = torch.empty(B, dtype=torch.float32, device="cuda")
    d_lse = torch.empty(B, dtype=torch.float32, device="cuda")

    def step(s):
        ctx.lzw_decode(new_codes[s], None, None, d_ntok, d_st, api.APPEND)
        ctx.hyper_embed(d_E, d_W, None, max_new=1)      # the step adds at most one entry per sequence
        ctx.set_option(api.OPT_TIMING, 1)      # HIP events around the decode kernel, on this stream
        ctx.extended_logits(d_H, 1, d_E, d_W, d_am, d_mx, d_lse, None)
        ctx.set_option(api.OPT_TIMING, 0)

    for s in range(args.warmup):
        step(s)
    torch.cuda.synchronize()
    ctx.read_timing()
    t0 = time.perf_counter()
    for s in range(args.warmup, n_steps):
        step(s)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    k_ms, k_n = ctx.read_timing()
    assert k_n == timed
    assert int(d_st.abs().sum()) == 0

    # the same steps captured once in a HIP graph (no event bracketing inside) and replayed: what a
    # serving loop that cannot afford a host round trip per kernel would run
    def step_plain(s):
        ctx.lzw_decode(new_codes[s], None, None, d_ntok, d_st, api.APPEND)
        ctx.hyper_embed(d_E, d_W, None, max_new=1)
        ctx.extended_logits(d_H, 1, d_E, d_W, d_am, d_mx, d_lse, None)

    am_eager = d_am.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for s in range(args.warmup, n_steps):
            step_plain(s)
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    graph.replay()
    torch.cuda.synchronize()
    graph_us = (time.perf_counter() - t0) * 1e6 / timed
    assert int(d_st.abs().sum()) == 0 and torch.equal(d_am, am_eager), "graph replay differs from the eager steps"

    # the same step with the pick drawn at a temperature (z2z_extended_sample) instead of the maximum
    d_lp = torch.empty(B, dtype=torch.float32, device="cuda")

    def step_sampled(s):
        ctx.lzw_decode(new_codes[s], None, None, d_ntok, d_st, api.APPEND)
        ctx.hyper_embed(d_E, d_W, None, max_new=1)
        ctx.extended_sample(d_H, 1, d_E, d_W, 0.8, 2506, s, d_am, d_lp)

    for s in range(args.warmup):
        step_sampled(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.warmup, n_steps):
        step_sampled(s)
    torch.cuda.synchronize()
    sample_us = (time.perf_counter() - t0) * 1e6 / timed
    assert int(d_st.abs().sum()) == 0

    # ... and with the top-k / nucleus filters in front of the draw (the logits go through library scratch)
    def step_filtered(s):
        ctx.lzw_decode(new_codes[s], None, None, d_ntok, d_st, api.APPEND)
        ctx.hyper_embed(d_E, d_W, None, max_new=1)
        ctx.extended_sample(d_H, 1, d_E, d_W, 0.8, 2506, s, d_am, d_lp, top_k=50, top_p=0.9)

    for s in range(args.warmup):
        step_filtered(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.warmup, n_steps):
        step_filtered(s)
    torch.cuda.synchronize()
    filtered_us = (time.perf_counter() - t0) * 1e6 / timed
    assert int(d_st.abs().sum()) == 0

    # ... and with the learned hyper-encoder (2 transformer layers, d_ff = 4 d) keeping the cache current
    # instead of the averaging one: the newest entry of every sequence goes through it each step
    enc = wl.make_encoder(cfg, n_layers=2, n_heads=32)
    layers = [{k: (to_device_bf16(torch, v) if k.startswith("w_") else torch.from_numpy(v).cuda()) for k, v in lay.items()}
              for lay in enc["layers"]]
    d_enc = api.Encoder(dict(n_heads=enc["n_heads"], attention_only=False, d_ff=enc["d_ff"],
                             pos=to_device_bf16(torch, enc["pos"]), layers=layers), torch.bfloat16)

    def step_learned(s):
        ctx.lzw_decode(new_codes[s], None, None, d_ntok, d_st, api.APPEND)
        ctx.hyper_encode(d_E, d_enc, d_W, None, max_new=1)
        ctx.extended_logits(d_H, 1, d_E, d_W, d_am, d_mx, d_lse, None)

    for s in range(args.warmup):
        step_learned(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.warmup, n_steps):
        step_learned(s)
    torch.cuda.synchronize()
    learned_us = (time.perf_counter() - t0) * 1e6 / timed
    assert int(d_st.abs().sum()) == 0
    # the same steps as one HIP graph (the newest-entry pass of the encoder is some 25 short kernels per step)
    am_learned = d_am.clone()
    side2 = torch.cuda.Stream()
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph2, stream=side2):
        for s in range(args.warmup, n_steps):
            step_learned(s)
    graph2.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    graph2.replay()
    torch.cuda.synchronize()
    learned_graph_us = (time.perf_counter() - t0) * 1e6 / timed
    assert int(d_st.abs().sum()) == 0 and torch.equal(d_am, am_learned), "graph replay differs from the eager steps"

    sizes = size_view.cpu().numpy()
    us = dt * 1e6 / timed
    bytes_step = 2.0 * d * (V + float(sizes.sum())) + 2.0 * B * d
    gbs = bytes_step / (us * 1e-6) / 1e9
    ctx.close()
    k_us = k_ms * 1e3 / k_n
    k_gbs = bytes_step / (k_us * 1e-6) / 1e9
    return dict(workload=cfg["name"], steps=timed, us_per_step=us, graph_us_per_step=graph_us,
                graph_frac=bytes_step / (graph_us * 1e-6) / 1e9 / PEAK_HBM_GBS,
                sample_topk50_topp09_us_per_step=filtered_us, learned_encoder_us_per_step=learned_us, learned_encoder_graph_us_per_step=learned_graph_us,
                sample_us_per_step=sample_us, sample_frac=bytes_step / (sample_us * 1e-6) / 1e9 / PEAK_HBM_GBS, algorithmic_bytes=bytes_step, achieved_GBs=gbs,
                peak_GBs=PEAK_HBM_GBS, frac=gbs / PEAK_HBM_GBS, mean_codebook_size=float(sizes.mean()),
                roofline={"bound": "hbm", "kernel": "logits_decode_kernel (64 rows, config 3)", "achieved": k_gbs,
                          "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": k_gbs / PEAK_HBM_GBS,
                          "traffic": TRAFFIC_BYTES.get("logits_decode_kernel@c3"), "avg_kernel_us": k_us,
                          "bytes_per_launch": bytes_step})


def run_encoder_workload(args, torch, api, wl):
    """Configuration 2 with the learned hyper-encoder in place of the averaging one: all 8 x 2048 entries
    through a two-layer transformer encoder (32 heads, d_ff = 4 d, random-init parameters), then the update of
    a generation step (the newest entry of every sequence only)."""
    cfg = wl.CONFIGS["c2"]
    B, N, V, M, cap, d = (cfg[k] for k in ("B", "N", "V", "M", "cap", "d"))
    t0 = time.time()
    enc = wl.make_encoder(cfg, n_layers=2, n_heads=32)
    log(f"[bench] encoder parameters generated in {time.time() - t0:.1f}s")
    layers = [{k: (to_device_bf16(torch, v) if k.startswith("w_") else torch.from_numpy(v).cuda()) for k, v in lay.items()}
              for lay in enc["layers"]]
    d_enc = api.Encoder(dict(n_heads=enc["n_heads"], attention_only=False, d_ff=enc["d_ff"],
                             pos=to_device_bf16(torch, enc["pos"]), layers=layers), torch.bfloat16)
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype="bf16")
    i32 = dict(dtype=torch.int32, device="cuda")
    d_tok = torch.from_numpy(wl.make_tokens(cfg)).cuda()
    d_codes, d_n, d_st = torch.empty((B, N), **i32), torch.empty(B, **i32), torch.empty(B, **i32)
    ctx.lzw_encode(d_tok, None, d_codes, d_n, d_st, api.RESET)
    d_E = to_device_bf16(torch, wl.make_embeddings(cfg))
    d_W = torch.empty((B, cap, d), dtype=torch.bfloat16, device="cuda")
    sizes = ctx.codebook()[2].cpu().numpy()

    def timed(reps, **kw):
        ctx.hyper_encode(d_E, d_enc, d_W, **kw)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            ctx.hyper_encode(d_E, d_enc, d_W, **kw)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    ms_full = timed(3)
    ms_inc = timed(20, first=None, max_new=1)
    rows = int(ctx.codebook()[1].sum().item())        # real slots of the existing entries = rows of the dense layers
    flops = 2.0 * rows * 2 * (4 * d * d + 2 * d * enc["d_ff"])
    weight_bytes = 2 * 2.0 * (4 * d * d + 2 * d * enc["d_ff"])
    # the encoder's gradient (training f_phi): forward again with every layer's rows kept, then reverse mode;
    # three dense products per dense layer (forward, input gradient, weight gradient)
    d_grad = api.Encoder(dict(n_heads=enc["n_heads"], attention_only=False, d_ff=enc["d_ff"],
                              pos=torch.empty_like(d_enc.params["pos"]),
                              layers=[{k: torch.empty_like(v) for k, v in lay.items()} for lay in layers]),
                         torch.bfloat16)
    d_dW = torch.randn((B, cap, d), device="cuda").to(torch.bfloat16)
    d_dE = torch.zeros((V, d), dtype=torch.float32, device="cuda")
    ctx.hyper_encode_backward(d_E, d_enc, d_dW, d_grad, d_dE)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(3):
        ctx.hyper_encode_backward(d_E, d_enc, d_dW, d_grad, d_dE)
    b.record()
    torch.cuda.synchronize()
    ms_bwd = a.elapsed_time(b) / 3
    # the same with the rows of a keeping forward call (a training step runs the forward once)
    ctx.hyper_encode_keep(d_E, d_enc, d_W)
    ctx.hyper_encode_backward(d_E, d_enc, d_dW, d_grad, d_dE, kept=True)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ms_keep = ms_kept_bwd = 0.0
    for _ in range(3):
        ev[0].record()
        ctx.hyper_encode_keep(d_E, d_enc, d_W)
        ev[1].record()
        ctx.hyper_encode_backward(d_E, d_enc, d_dW, d_grad, d_dE, kept=True)
        ev[2].record()
        torch.cuda.synchronize()
        ms_keep += ev[0].elapsed_time(ev[1]) / 3
        ms_kept_bwd += ev[1].elapsed_time(ev[2]) / 3
    ctx.close()
    return {
        "workload": f"c2 codebooks ({int(sizes.sum())} entries, {rows} real slots of M={M}), learned hyper-encoder: 2 pre-norm "
                    f"transformer layers, 32 heads, d_ff={enc['d_ff']}, d={d} bf16",
        "full_ms": ms_full, "dense_flops": flops, "TFLOPs": flops / (ms_full * 1e-3) / 1e12,
        "frac_of_bf16_peak": flops / (ms_full * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "newest_entry_us": ms_inc * 1e3, "newest_entry_weight_bytes": weight_bytes,
        "newest_entry_GBs": weight_bytes / (ms_inc * 1e-3) / 1e9,
        "backward_ms": ms_bwd, "backward_dense_flops": 3 * flops,
        "backward_TFLOPs": 3 * flops / (ms_bwd * 1e-3) / 1e12,
        "keeping_forward_ms": ms_keep, "backward_on_kept_rows_ms": ms_kept_bwd,
        "backward_on_kept_rows_TFLOPs": 2 * flops / (ms_kept_bwd * 1e-3) / 1e12,
    }


def run_backward_workload(args, torch, api, wl):
    """Configuration 2 as a training step of the unembedding: the loss of every position's next code
    (extended_nll), its gradient into H, W_base, W_hyper (extended_nll_backward) and through the pooling."""
    cfg = wl.CONFIGS["c2"]
    B, N, V, M, cap, d = (cfg[k] for k in ("B", "N", "V", "M", "cap", "d"))
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype="bf16")
    i32 = dict(dtype=torch.int32, device="cuda")
    d_tok = torch.from_numpy(wl.make_tokens(cfg)).cuda()
    d_codes, d_n, d_st = torch.full((B, N), -1, **i32), torch.empty(B, **i32), torch.empty(B, **i32)
    ctx.lzw_encode(d_tok, None, d_codes, d_n, d_st, api.RESET)
    d_E = to_device_bf16(torch, wl.make_embeddings(cfg))
    d_H = to_device_bf16(torch, wl.make_hidden(cfg, B * N))
    d_W = torch.empty((B, cap, d), dtype=torch.bfloat16, device="cuda")
    ctx.hyper_embed(d_E, d_W)
    # row i of a sequence is asked for code i + 1 of its compressed stream; rows past the stream have no target
    d_t = torch.roll(d_codes, -1, dims=1).contiguous()
    d_t[:, -1] = -1
    d_t = d_t.reshape(-1)
    nll = torch.empty(B * N, dtype=torch.float32, device="cuda")
    lse = torch.empty_like(nll)
    dH, dWb, dWh = torch.empty_like(d_H), torch.empty_like(d_E), torch.empty_like(d_W)
    dE = torch.zeros((V, d), dtype=torch.float32, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    fwd, bwd, pool = [], [], []
    for rep in range(4):                               # the first one sizes the work space
        ev[0].record()
        ctx.extended_nll(d_H, N, d_E, d_W, d_t, nll, lse)
        ev[1].record()
        ctx.extended_nll_backward(d_H, N, d_E, d_W, d_t, lse, None, dH, dWb, dWh)
        ev[2].record()
        ctx.hyper_embed_backward(dWh, dE)
        ev[3].record()
        torch.cuda.synchronize()
        if rep > 0:
            fwd.append(ev[0].elapsed_time(ev[1]))
            bwd.append(ev[1].elapsed_time(ev[2]))
            pool.append(ev[2].elapsed_time(ev[3]))
    sizes = ctx.codebook()[2].cpu().numpy()
    cols = V + float(sizes.mean())
    flops_bwd = 3 * 2.0 * B * N * d * cols           # the logits again, dH, dW
    n_targets = int((d_t >= 0).sum().item())
    mean_nll = float(nll[torch.isfinite(nll) & (d_t >= 0)].mean().item())
    ctx.close()
    ms = lambda v: sum(v) / len(v)
    return {
        "workload": f"c2: {B * N} rows x {int(cols)} columns, d={d} bf16; targets = the next code of the compressed stream "
                    f"({n_targets} rows with a target)",
        "forward_nll_ms": ms(fwd), "backward_ms": ms(bwd), "pooling_backward_ms": ms(pool),
        "backward_flops": flops_bwd, "backward_TFLOPs": flops_bwd / (ms(bwd) * 1e-3) / 1e12,
        "backward_frac_of_bf16_peak": flops_bwd / (ms(bwd) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "mean_nll": mean_nll,
    }


def cpu_baseline(wl, host, budget_rows=4096):
    """The oracle, as it stands, on the host cores: LZW and pooling on the full configuration-2 batch, the
    joint logits on a sample of rows of sequence 0 (all columns); combined into tokens/s of the whole step."""
    import numpy as np

    import oracle

    cfg = wl.CONFIGS["c2"]
    B, N, V, M, cap = (cfg[k] for k in ("B", "N", "V", "M", "cap"))
    tokens, E, H = host["tokens"], host["E"], host["H"]
    t0 = time.perf_counter()
    enc = [oracle.lzw_encode(tokens[b].tolist(), V, M, cap) for b in range(B)]
    for b in range(B):
        back, _, _ = oracle.lzw_decode(enc[b][0], V, M, cap)
        assert back == tokens[b].tolist()
    t_lzw = time.perf_counter() - t0
    t0 = time.perf_counter()
    W0 = oracle.hyper_embed(E, "bf16", enc[0][1], cap, "mean")
    t_embed = (time.perf_counter() - t0) * B                      # one sequence timed, B alike
    t0 = time.perf_counter()
    oracle.extended_logits(H[:budget_rows], E, W0, len(enc[0][1]), "bf16", return_logits=False)
    t_rows = time.perf_counter() - t0
    per_token = (t_lzw + t_embed) / (B * N) + t_rows / budget_rows
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    return dict(value=1.0 / per_token, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=(f"config 2: LZW encode+decode of all {B * N} tokens ({t_lzw:.2f}s, 1 thread), mean pooling "
                        f"of one sequence's {len(enc[0][1])} entries x{B} ({t_embed:.2f}s), joint logits+softmax of "
                        f"{budget_rows} rows of sequence 0 over all {V + len(enc[0][1])} columns in float64 "
                        f"({t_rows:.2f}s, BLAS threads); per-token costs summed"),
                host_cpus=os.cpu_count())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-encoder", action="store_true", help="skip the learned hyper-encoder measurement")
    ap.add_argument("--no-backward", action="store_true", help="skip the loss forward + backward measurement")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known traffic, to scale the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2506_01084_amd import api, workloads as wl

    torch.cuda.set_device(0)
    api.load_library()
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    res, host = run_prefill_workload(args, torch, api, wl)
    assert res["kernel_launches"] == args.steps
    k_ms = res["kernel_ms_total"] / res["kernel_launches"]
    log(f"[bench] step {res['ms_per_step']:.2f} ms; stages {res['stage_ms']}; base-part kernel {k_ms:.3f} ms")
    dec = None if args.no_decode else run_decode_workload(args, torch, api, wl)
    enc = None if args.no_encoder else run_encoder_workload(args, torch, api, wl)
    bwd = None if args.no_backward else run_backward_workload(args, torch, api, wl)
    cpu = None if args.no_cpu_baseline else cpu_baseline(wl, host)

    cfg = res["cfg"]
    achieved = res["flops_base"] / (k_ms * 1e-3) / 1e12
    st = res["stage_ms"]
    line = {
        "metric": "base tokens/s LZW+hyper_embed; extended_logits TFLOP/s & decode-step µs",
        "value": res["tokens"] / (res["ms_per_step"] * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg['name']}: B={cfg['B']} x N={cfg['N']} tokens, V={cfg['V']}, d={cfg['d']} bf16, "
                               f"M={cfg['M']}, cap={cfg['cap']}, mean pooling, logits for all {res['tokens']} rows "
                               f"over V+C_b columns, plus one generation step and the final decompression"},
        "submetrics": {
            "lzw_encode_plus_hyper_embed_tokens_per_s": res["tokens"] / ((st["lzw_encode"] + st["hyper_embed"]) * 1e-3),
            "extended_logits_TFLOPs": res["flops_all"] / (st["extended_logits"] * 1e-3) / 1e12,
            "decode_step_us": None if dec is None else dec["us_per_step"],
            "stage_ms": st,
            "mean_codebook_size": sum(res["sizes"]) / len(res["sizes"]),
            "compression_rate": sum(res["n_codes"]) / res["tokens"],
            "entries_reused_frac": res["entries_reused_frac"],
        },
        "roofline": {"bound": "mfma", "kernel": "logits_fast_kernel<0> (base-vocabulary part of the prefill extended_logits call)",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": TRAFFIC_BYTES.get("logits_fast_kernel<0>@c2"),
                     "avg_kernel_ms": k_ms, "flops_per_launch": res["flops_base"]},
        "cpu_baseline": cpu,
        "decode_step": dec,
        "hyper_encode": enc,
        "nll_backward": bwd,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
