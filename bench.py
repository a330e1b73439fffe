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
The other prefill configurations (1: tiny fp32; 4: long code-like context; 5: large vocabulary, deep merges,
weighted pooling) run the same stages a few times each and are reported in `prefill_configs`, with a roofline
object per extended_logits kernel; configuration 2 is also run with one hidden row per compressed position
(`c2_compressed_rows`).
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

PEAK_F32_TFLOPS = 157.3        # MI355X dense fp32 MFMA


def load_traffic_table():
    """HBM bytes per launch (fetch + write) of the dominant kernels, measured by the rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE runs summarised under profiles/.  profiles/hbm_traffic.txt holds one line per kernel and workload:
    key, bytes, the sha256 (first 16 hex digits) of the kernel's sources at the time of the run, the commit and
    the summary file.  A line whose source hash no longer matches the tree is stale and reads as None."""
    import hashlib

    table = {}
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return table
    for line in open(path):
        line = line.split("#", 1)[0].strip()
        if not line:
            continue
        key, nbytes, digest, sources = line.split()[:4]
        h = hashlib.sha256()
        for src in sources.split(","):
            with open(os.path.join(ROOT, "paper_2506_01084_amd", "csrc", src), "rb") as f:
                h.update(f.read())
        table[key] = float(nbytes) if h.hexdigest()[:16] == digest else None
    return table


TRAFFIC_BYTES = load_traffic_table()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def to_device_bf16(torch, bits, dtype="bf16"):
    """Host array in the storage format (uint16 bf16 bit patterns, or float32) -> device tensor (memory plumbing
    only)."""
    import numpy as np

    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.float32)).cuda()
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


def run_prefill_workload(args, torch, api, wl, name="c2", steps=None, warmup=None, compressed_rows=False):
    """One configuration through the whole path, `steps` times after `warmup`; stage times from events on the
    stream, the base-vocabulary logits kernel bracketed by the library's own events.  compressed_rows: afterwards
    also time extended_logits with one hidden row per compressed position (max_b n_codes rows per sequence)."""
    steps = args.steps if steps is None else steps
    warmup = args.warmup if warmup is None else warmup
    cfg = wl.CONFIGS[name]
    B, N, V, M, cap, d = (cfg[k] for k in ("B", "N", "V", "M", "cap", "d"))
    dt_name = cfg["dtype"]
    tdt = torch.float32 if dt_name == "f32" else torch.bfloat16
    rows = B * N
    t0 = time.time()
    tokens = wl.make_tokens(cfg)
    E = wl.make_embeddings(cfg)
    H = wl.make_hidden(cfg, rows)
    log(f"[bench] {name} inputs generated in {time.time() - t0:.1f}s")
    d_tok = torch.from_numpy(tokens).cuda()
    d_E = to_device_bf16(torch, E, dt_name)         # tied: the matrix pooled is the LM head
    d_H = to_device_bf16(torch, H, dt_name)
    d_Hdec = d_H[N - 1::N].contiguous()             # one hidden row per sequence for the generation step
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=d, dtype=dt_name, pool=cfg["pool"],
                      w=wl.make_pool_weights(cfg).tolist())
    if getattr(args, "probe", "none") != "none":
        ctx.set_option(api.OPT_LOGITS_KERNEL, {"noreq": 2, "mfma": 3}[args.probe])
    if getattr(args, "logits_map", 0):
        ctx.set_option(api.OPT_LOGITS_MAP, args.logits_map)
    i32 = dict(dtype=torch.int32, device="cuda")
    d_codes = torch.empty((B, N), **i32)
    d_ncodes = torch.empty(B, **i32)
    d_status = torch.empty(B, **i32)
    d_W = torch.empty((B, cap, d), dtype=tdt, device="cuda")
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
            ctx.step_update(d_am[N - 1:], d_E, d_W, d_ntok1, d_st1, stride=N)
            ctx.extended_logits(d_Hdec, 1, d_E, d_W, d_am1, d_mx1, d_lse1, None)
        with stages["lzw_decode"]:
            ctx.lzw_decode(d_codes, d_ncodes, d_back, d_nback, d_st2, api.RESET)

    stages = {n: Stage(torch, warmup) for n in names}
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ctx.read_timing()
    stages = {n: Stage(torch, steps) for n in names}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_ms, launches = ctx.read_timing()
    counts = ctx.read_launches()

    # sanity inside the bench: statuses clean, round trip exact
    assert int(d_status.abs().sum()) == 0 and int(d_st1.abs().sum()) == 0 and int(d_st2.abs().sum()) == 0
    assert torch.equal(d_back, d_tok), "lzw_decode(lzw_encode(x)) != x"
    sizes = size_view.cpu().numpy()
    ncodes = d_ncodes.cpu().numpy()
    # how many of the entries the code stream ever names (the paper's discussion: about a quarter on its data)
    d_usage = torch.zeros((B, cap), **i32)
    ctx.codebook_usage(d_codes, d_ncodes, d_usage)
    reused = float((d_usage > 0).sum().item()) / max(1.0, float(sizes.sum()))

    # rounds of the parse kernels (the serial chain of a call), read from the library's own counters
    ctx.lzw_encode(d_tok, None, d_codes, d_ncodes, d_status, api.RESET)
    torch.cuda.synchronize()
    rounds_enc = ctx.lzw_rounds().cpu().numpy().copy()
    ctx.lzw_decode(d_codes, d_ncodes, d_back, d_nback, d_st2, api.RESET)
    torch.cuda.synchronize()
    rounds_dec = ctx.lzw_rounds().cpu().numpy().copy()

    ms_per_step = dt * 1e3 / steps
    stage_ms = {n: stages[n].total_ms() / steps for n in names}
    flops_base = 2.0 * rows * d * V
    flops_all = 2.0 * rows * d * (V + float(sizes.mean()))        # the columns that exist: V + C_b, not V + cap
    # bytes hyper_embed has to move: every entry's constituent rows in and its pooled row out
    ent_len = ctx.codebook()[1]
    embed_bytes = float((ent_len.sum().item() + int(sizes.sum())) * d * (4 if dt_name == "f32" else 2))
    out = dict(ms_per_step=ms_per_step, stage_ms=stage_ms, kernel_ms_total=kernel_ms, kernel_launches=launches,
               flops_base=flops_base, flops_all=flops_all, sizes=sizes.tolist(), n_codes=ncodes.tolist(),
               tokens=B * N, cfg=cfg, entries_reused_frac=reused, steps=steps, embed_bytes=embed_bytes,
               tile_kernel=counts["tile_base"] > 0, rounds_enc=rounds_enc.tolist(), rounds_dec=rounds_dec.tolist())
    if compressed_rows:
        # one hidden row per compressed position: what a model running on the compressed sequence would hand
        # over (section 2.4).  Rows per sequence are uniform in the call, so the longest code stream sets them.
        rps = int(ncodes.max())
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ctx.extended_logits(d_H[:B * rps], rps, d_E, d_W, d_am[:B * rps], d_mx[:B * rps], d_lse[:B * rps], None)
        ev[0].record()
        for _ in range(steps):
            ctx.extended_logits(d_H[:B * rps], rps, d_E, d_W, d_am[:B * rps], d_mx[:B * rps], d_lse[:B * rps], None)
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / steps
        fl = 2.0 * B * rps * d * (V + float(sizes.mean()))
        out["compressed_rows"] = dict(rows_per_seq=rps, rows=B * rps, sum_n_codes=int(ncodes.sum()),
                                      extended_logits_ms=ms, flops=fl, TFLOPs=fl / (ms * 1e-3) / 1e12,
                                      frac_of_bf16_peak=fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS)
    host = dict(tokens=tokens, E=E, H=H)
    ctx.close()
    return out, host


def config_report(res):
    """The per-configuration object of the JSON line: stage times, the metric's rates, and the roofline of the
    extended_logits base-vocabulary kernel of that configuration."""
    cfg, st = res["cfg"], res["stage_ms"]
    k_ms = res["kernel_ms_total"] / max(res["kernel_launches"], 1)
    bf16 = cfg["dtype"] == "bf16"
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_TFLOPS
    achieved = res["flops_base"] / (k_ms * 1e-3) / 1e12
    whole = res["flops_all"] / (st["extended_logits"] * 1e-3) / 1e12
    kernel = ("logits_fast_kernel<0>" if res["tile_kernel"] else
              "logits_general_kernel (fp32 MFMA)" if not bf16 else "logits_general_kernel")
    return {
        "workload": f"{cfg['name']}: B={cfg['B']} x N={cfg['N']}, V={cfg['V']}, d={cfg['d']} {cfg['dtype']}, M={cfg['M']}, "
                    f"cap={cfg['cap']}, {cfg['pool']} pooling",
        "steps": res["steps"], "tokens": res["tokens"], "stage_ms": st,
        "lzw_encode_tokens_per_s": res["tokens"] / (st["lzw_encode"] * 1e-3),
        "lzw_decode_tokens_per_s": res["tokens"] / (st["lzw_decode"] * 1e-3),
        "lzw_encode_plus_hyper_embed_tokens_per_s": res["tokens"] / ((st["lzw_encode"] + st["hyper_embed"]) * 1e-3),
        # the parse is a serial chain per sequence: its time is (rounds of the longest sequence) x (time per round);
        # cycles are quoted at the 2.4 GHz peak clock
        "lzw": {"encode_rounds_max": max(res["rounds_enc"]), "decode_rounds_max": max(res["rounds_dec"]),
                "encode_us_per_round": st["lzw_encode"] * 1e3 / max(res["rounds_enc"]),
                "decode_us_per_round": st["lzw_decode"] * 1e3 / max(res["rounds_dec"]),
                "encode_cycles_per_token_of_a_sequence_at_2p4GHz": st["lzw_encode"] * 1e-3 * 2.4e9 / cfg["N"],
                "decode_cycles_per_token_of_a_sequence_at_2p4GHz": st["lzw_decode"] * 1e-3 * 2.4e9 / cfg["N"],
                "tokens_per_round_encode": cfg["N"] / (sum(res["rounds_enc"]) / len(res["rounds_enc"]))},
        "hyper_embed_algorithmic_bytes": res["embed_bytes"],
        "hyper_embed_algorithmic_GBs": res["embed_bytes"] / (st["hyper_embed"] * 1e-3) / 1e9,
        "sum_codebook_sizes": int(sum(res["sizes"])), "compression_rate": sum(res["n_codes"]) / res["tokens"],
        "extended_logits_ms": st["extended_logits"], "extended_logits_TFLOPs": whole,
        "roofline": {"bound": "mfma", "kernel": kernel + " (base-vocabulary part)", "achieved": achieved, "peak": peak,
                     "unit": "TFLOP/s", "frac": achieved / peak, "avg_kernel_ms": k_ms,
                     "flops_per_launch": res["flops_base"], "whole_call_achieved": whole,
                     "whole_call_frac": whole / peak,
                     "traffic": TRAFFIC_BYTES.get(f"logits_fast_kernel<0>@{cfg['name'][:2]}")},
    }


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
        ctx.step_update(new_codes[s], d_E, d_W, d_ntok, d_st)      # codebook update + the new entry's cache row
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
        ctx.step_update(new_codes[s], d_E, d_W, d_ntok, d_st)
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
        ctx.step_update(new_codes[s], d_E, d_W, d_ntok, d_st)
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
        ctx.step_update(new_codes[s], d_E, d_W, d_ntok, d_st)
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
                sample_us_per_step=sample_us, sample_frac=bytes_step / (sample_us * 1e-6) / 1e9 / PEAK_HBM_GBS,
                sample_topk50_topp09_frac=bytes_step / (filtered_us * 1e-6) / 1e9 / PEAK_HBM_GBS,
                learned_encoder_frac=bytes_step / (learned_us * 1e-6) / 1e9 / PEAK_HBM_GBS, algorithmic_bytes=bytes_step, achieved_GBs=gbs,
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


def run_lzw_batch(args, torch, api, wl, B=2048):
    """Many documents per call (the preprocessing case): B sequences of configuration 2's kind through
    lzw_encode and lzw_decode; one wave per sequence, tables in global memory."""
    cfg = wl.scaled(wl.CONFIGS["c2"], B=B, seed=2900)
    N, V, M, cap = cfg["N"], cfg["V"], cfg["M"], cfg["cap"]
    t0 = time.time()
    d_tok = torch.from_numpy(wl.make_tokens(cfg)).cuda()
    log(f"[bench] {B} x {N} tokens generated in {time.time() - t0:.1f}s")
    ctx = api.Context(B=B, V=V, M=M, cap=cap, d=64, dtype="bf16", pool="mean")
    i32 = dict(dtype=torch.int32, device="cuda")
    d_codes, d_n, d_st = torch.empty((B, N), **i32), torch.empty(B, **i32), torch.empty(B, **i32)
    d_back, d_nb, d_st2 = torch.empty((B, N), **i32), torch.empty(B, **i32), torch.empty(B, **i32)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    enc, dec = [], []
    for rep in range(6):
        ev[0].record()
        ctx.lzw_encode(d_tok, None, d_codes, d_n, d_st, api.RESET)
        ev[1].record()
        ctx.lzw_decode(d_codes, d_n, d_back, d_nb, d_st2, api.RESET)
        ev[2].record()
        torch.cuda.synchronize()
        if rep:
            enc.append(ev[0].elapsed_time(ev[1]))
            dec.append(ev[1].elapsed_time(ev[2]))
    assert int(d_st.abs().sum()) == 0 and int(d_st2.abs().sum()) == 0 and torch.equal(d_back, d_tok)
    rounds_dec = int(ctx.lzw_rounds().max().item())
    ctx.lzw_encode(d_tok, None, d_codes, d_n, d_st, api.RESET)
    torch.cuda.synchronize()
    rounds_enc = int(ctx.lzw_rounds().max().item())
    ctx.close()
    e, d_ = sum(enc) / len(enc), sum(dec) / len(dec)
    return dict(workload=f"{B} sequences x {N} tokens, V={V}, M={M}, cap={cap} (configuration 2's generator)",
                tokens=B * N, encode_ms=e, decode_ms=d_, encode_tokens_per_s=B * N / (e * 1e-3),
                decode_tokens_per_s=B * N / (d_ * 1e-3), encode_rounds_max=rounds_enc, decode_rounds_max=rounds_dec,
                encode_us_per_round=e * 1e3 / rounds_enc, decode_us_per_round=d_ * 1e3 / rounds_dec)


def _oracle_lzw_one(job):
    """Worker of the process-per-sequence oracle timing (imports the oracle only)."""
    import oracle

    toks, V, M, cap = job
    codes, entries, _ = oracle.lzw_encode(toks, V, M, cap)
    back, _, _ = oracle.lzw_decode(codes, V, M, cap)
    assert back == toks
    return len(codes)


def cpu_lzw_parallel(wl):
    """The LZW oracle on all of configuration 2, one process per sequence (up to the host's cores).  Runs before
    the GPU is touched: the workers are forked from a process that holds no GPU state."""
    import multiprocessing as mp

    cfg = wl.CONFIGS["c2"]
    tokens = wl.make_tokens(cfg)
    jobs = [(tokens[b].tolist(), cfg["V"], cfg["M"], cfg["cap"]) for b in range(cfg["B"])]
    n = max(1, min(cfg["B"], os.cpu_count() or 1))
    with mp.get_context("fork").Pool(n) as pool:
        pool.map(_oracle_lzw_one, jobs[:n])            # start-up and imports outside the timed part
        reps = 8                                       # each sequence several times: a single parse is ~2 ms
        t0 = time.perf_counter()
        pool.map(_oracle_lzw_one, jobs * reps, chunksize=reps)
        dt = time.perf_counter() - t0
    return dict(seconds=dt, processes=n, tokens=reps * cfg["B"] * cfg["N"])


def cpu_baseline(wl, host, lzw_par, budget_rows=4096):
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
    out = dict(value=1.0 / per_token, unit="tokens/s", cores=int(threads), kind="oracle",
               sample=(f"config 2: LZW encode+decode of all {B * N} tokens ({t_lzw:.2f}s, 1 thread), mean pooling "
                       f"of one sequence's {len(enc[0][1])} entries x{B} ({t_embed:.2f}s), joint logits+softmax of "
                       f"{budget_rows} rows of sequence 0 over all {V + len(enc[0][1])} columns in float64 "
                       f"({t_rows:.2f}s, BLAS threads); per-token costs summed"),
               host_cpus=os.cpu_count(),
               lzw_tokens_per_s_one_thread=B * N / t_lzw)
    if lzw_par is not None:
        out["lzw_tokens_per_s_process_per_sequence"] = lzw_par["tokens"] / lzw_par["seconds"]
        out["lzw_processes"] = lzw_par["processes"]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-encoder", action="store_true", help="skip the learned hyper-encoder measurement")
    ap.add_argument("--no-backward", action="store_true", help="skip the loss forward + backward measurement")
    ap.add_argument("--no-configs", action="store_true", help="skip configurations 1, 4 and 5")
    ap.add_argument("--only", default="", help="comma-separated configurations for the per-configuration part "
                                               "(default c1,c4,c5)")
    ap.add_argument("--probe", choices=["none", "noreq", "mfma"], default="none",
                    help="MEASUREMENT PROBE, not a benchmark: run configuration 2's base-vocabulary logits kernel "
                         "without operand requests (noreq) or as the MFMA stream alone (mfma); its outputs are not "
                         "the logits' reduction and the JSON line says so")
    ap.add_argument("--logits-map", type=lambda v: int(v, 0), default=0,
                    help="workgroup -> tile order of the base-vocabulary logits kernel (Z2Z_OPT_LOGITS_MAP), for sweeps")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known traffic, to scale the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    from paper_2506_01084_amd import workloads as wl

    if args.probe != "none":
        args.no_cpu_baseline = True
    lzw_par = None if args.no_cpu_baseline else cpu_lzw_parallel(wl)     # forks workers: before any GPU call

    if args.probe != "none":
        args.no_configs = args.no_decode = args.no_encoder = args.no_backward = True

    import torch

    from paper_2506_01084_amd import api

    torch.cuda.set_device(0)
    api.load_library()
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    res, host = run_prefill_workload(args, torch, api, wl, "c2", compressed_rows=True)
    assert res["kernel_launches"] == args.steps and res["tile_kernel"]
    k_ms = res["kernel_ms_total"] / res["kernel_launches"]
    log(f"[bench] step {res['ms_per_step']:.2f} ms; stages {res['stage_ms']}; base-part kernel {k_ms:.3f} ms")
    dec = None if args.no_decode else run_decode_workload(args, torch, api, wl)
    enc = None if args.no_encoder else run_encoder_workload(args, torch, api, wl)
    bwd = None if args.no_backward else run_backward_workload(args, torch, api, wl)
    lzw_batch = None if args.no_configs else run_lzw_batch(args, torch, api, wl)
    cpu = None if args.no_cpu_baseline else cpu_baseline(wl, host, lzw_par)
    del host
    per_config = {"c2": config_report(res)}
    per_config["c2"]["compressed_rows"] = res.get("compressed_rows")
    if not args.no_configs:
        # the other prefill configurations: a few passes each (config 5's logits alone are ~0.25 s per pass)
        for name in [n for n in (args.only.split(",") if args.only else ["c1", "c4", "c5"]) if n]:
            n_steps = {"c1": 20, "c4": 5, "c5": 3}.get(name, 3)
            r, h = run_prefill_workload(args, torch, api, wl, name, steps=n_steps, warmup=1)
            del h
            per_config[name] = config_report(r)
            log(f"[bench] {name}: stages {r['stage_ms']}; logits {per_config[name]['extended_logits_TFLOPs']:.1f} TFLOP/s")
            torch.cuda.empty_cache()

    cfg = res["cfg"]
    achieved = res["flops_base"] / (k_ms * 1e-3) / 1e12
    st = res["stage_ms"]
    probe = args.probe != "none"
    line = {
        "metric": ("PROBE (not a result): the logits kernel ran in measurement mode '%s'" % args.probe) if probe else
                  "base tokens/s LZW+hyper_embed; extended_logits TFLOP/s & decode-step µs",
        "value": None if probe else res["tokens"] / (res["ms_per_step"] * 1e-3),
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
                     "avg_kernel_ms": k_ms, "flops_per_launch": res["flops_base"],
                     "whole_call_achieved": res["flops_all"] / (st["extended_logits"] * 1e-3) / 1e12,
                     "whole_call_frac": res["flops_all"] / (st["extended_logits"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        "prefill_configs": per_config,
        "lzw_batch": lzw_batch,
        "cpu_baseline": cpu,
        "decode_step": dec,
        "hyper_encode": enc,
        "nll_backward": bwd,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
