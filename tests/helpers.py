"""Shared helpers for the GPU parity tests: run the HIP path through the binding, run the oracle, compare."""
from __future__ import annotations

import numpy as np

import oracle


def torch_storage(arr: np.ndarray, dtype: str):
    """Host array in the storage format (float32, or bf16 bit patterns as uint16) -> device tensor."""
    import torch

    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda()
    t = torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).cuda()
    return t.view(torch.bfloat16)


def storage_to_host(t, dtype: str) -> np.ndarray:
    """Device tensor -> host array in the storage format."""
    import torch

    if dtype == "f32":
        return t.detach().cpu().numpy()
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def oracle_encode_batch(tokens: np.ndarray, lens: np.ndarray, V: int, M: int, cap: int):
    """Per-sequence oracle encode: list of (codes, entries, status)."""
    return [oracle.lzw_encode(tokens[b, : int(lens[b])].tolist(), V, M, cap) for b in range(tokens.shape[0])]


def gpu_encode(ctx, tokens: np.ndarray, lens=None, out_stride=None, flags=1):
    """Run lzw_encode; returns host arrays (codes [B, out_stride], n_codes [B], status [B])."""
    import torch

    B, N = tokens.shape
    out_stride = N if out_stride is None else out_stride
    d_tok = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).cuda()
    d_len = None if lens is None else torch.from_numpy(np.ascontiguousarray(lens, dtype=np.int32)).cuda()
    d_codes = torch.full((B, max(out_stride, 1)), -7, dtype=torch.int32, device="cuda")[:, :out_stride].contiguous()
    d_n = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    d_st = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ctx.lzw_encode(d_tok, d_len, d_codes, d_n, d_st, flags)
    torch.cuda.synchronize()
    return d_codes.cpu().numpy(), d_n.cpu().numpy(), d_st.cpu().numpy()


def gpu_decode(ctx, codes: np.ndarray, n_codes=None, out_stride=0, flags=1):
    import torch

    B = codes.shape[0]
    d_codes = torch.from_numpy(np.ascontiguousarray(codes, dtype=np.int32)).cuda()
    d_nc = None if n_codes is None else torch.from_numpy(np.ascontiguousarray(n_codes, dtype=np.int32)).cuda()
    d_tok = None
    if out_stride > 0:
        d_tok = torch.full((B, out_stride), -7, dtype=torch.int32, device="cuda")
    d_n = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    d_st = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ctx.lzw_decode(d_codes, d_nc, d_tok, d_n, d_st, flags)
    torch.cuda.synchronize()
    return (None if d_tok is None else d_tok.cpu().numpy()), d_n.cpu().numpy(), d_st.cpu().numpy()


def assert_codebook_equal(ctx, ref_entries_per_seq, M: int, cap: int):
    """The context's codebook views against oracle entry lists, bit for bit (including padding)."""
    import torch

    torch.cuda.synchronize()
    ent, ln, size = (t.cpu().numpy() for t in ctx.codebook())
    for b, entries in enumerate(ref_entries_per_seq):
        tok, l, C = oracle.pack_entries(entries, cap, M)
        assert int(size[b]) == C, f"seq {b}: size {int(size[b])} != {C}"
        if cap:
            assert (ln[b] == l).all(), f"seq {b}: entry lengths differ"
            assert (ent[b] == tok).all(), f"seq {b}: entry tokens differ"


def hyper_embed_bound(E: np.ndarray, dtype: str, entries, pool: str, w, cap: int) -> np.ndarray:
    """[cap, d] sum_j a_j |E[t_j]|: the scale the rounding error of a pooled row is relative to."""
    d = E.shape[1]
    out = np.zeros((cap, d))
    for i, e in enumerate(entries):
        a = oracle.pool_coefficients(len(e), pool, w)
        for j, t in enumerate(e):
            out[i] += a[j] * np.abs(oracle.to_f64(E[t], dtype))
    return out


def check_logits_rows(ref: dict, argmax, mx, lse, logits=None, tol=2e-2, margin_min=1e-2, V=None):
    """Compare GPU per-row results against one oracle result dict (rows of one sequence).

    Bars: max_v |l_gpu - l_ref| / max_v |l_ref| <= tol per row (when full logits are given);
    |max - ref| <= tol * max(1, |ref|); |lse - ref| <= tol * max(1, |ref|);
    argmax identical wherever the oracle's top-2 gap exceeds margin_min.
    Returns the largest observed errors.
    """
    rmax, rlse, ram, margin = ref["max"], ref["lse"], ref["argmax"], ref["margin"]
    e_max = np.abs(mx.astype(np.float64) - rmax) / np.maximum(1.0, np.abs(rmax))
    e_lse = np.abs(lse.astype(np.float64) - rlse) / np.maximum(1.0, np.abs(rlse))
    assert (e_max <= tol).all(), f"max: {e_max.max()}"
    assert (e_lse <= tol).all(), f"lse: {e_lse.max()}"
    decided = margin > margin_min
    assert (argmax[decided] == ram[decided]).all(), "argmax differs where the top-2 gap is decisive"
    # undecided rows must still point at a logit within the gap of the maximum
    if (~decided).any() and "logits" in ref:
        idx = np.nonzero(~decided)[0]
        picked = ref["logits"][idx, argmax[idx]]
        assert (rmax[idx] - picked <= margin_min + 1e-6).all()
    e_log = 0.0
    if logits is not None:
        rl = ref["logits"]
        n = rl.shape[1]
        scale = np.abs(rl).max(axis=1)
        e = np.abs(logits[:, :n].astype(np.float64) - rl).max(axis=1) / scale
        assert (e <= tol).all(), f"logits: {e.max()}"
        e_log = float(e.max())
        if logits.shape[1] > n and V is not None:
            C = n - V
            assert np.isneginf(logits[:, V + C:]).all(), "unused hyper slots must read -inf"
    return dict(max=float(e_max.max()), lse=float(e_lse.max()), logits=e_log)


def encoder_to_device(enc: dict, dtype: str):
    """Host encoder parameters (workloads.make_encoder) -> the binding's Encoder over device tensors."""
    import torch
    from paper_2506_01084_amd import api

    layers = []
    for lay in enc["layers"]:
        layers.append({k: (torch_storage(v, dtype) if k.startswith("w_") else torch.from_numpy(v).cuda())
                       for k, v in lay.items()})
    params = dict(n_heads=enc["n_heads"], attention_only=enc["attention_only"], d_ff=enc["d_ff"],
                  pos=None if enc["pos"] is None else torch_storage(enc["pos"], dtype), layers=layers)
    return api.Encoder(params, torch.float32 if dtype == "f32" else torch.bfloat16)
