"""Thin ctypes binding of libz2z.so: argument marshalling only, every step runs in the HIP kernels.

PyTorch is used for device memory and streams (tensor.data_ptr(), the current stream's handle).
There is no CPU fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_float, c_int32, c_void_p
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libz2z.so")

F32, BF16 = 0, 1
POOL_MEAN, POOL_WEIGHTED = 0, 1
APPEND, RESET = 0, 1
ST_OK, ST_BAD_TOKEN, ST_BAD_CODE, ST_OVERFLOW = 0, 1, 2, 4
OPT_LOGITS_KERNEL, OPT_LOGITS_STRIP, OPT_LZW_KERNEL, OPT_DECODE_KERNEL, OPT_TIMING, OPT_LOGITS_MAP = 1, 2, 3, 4, 5, 6
OPT_SAMPLE_KERNEL = 7
OPT_BACKWARD_CHUNK = 8
MAX_M = 8
E_INVAL, E_NOMEM, E_HIP, E_UNSUPPORTED, E_LIMIT, E_CAPTURE = -1, -2, -3, -4, -5, -6
STATIC_PARTS = 1 << 22

ENC_KEPT = 1
EXPORTS = ["z2z_create", "z2z_destroy", "z2z_reset", "z2z_lzw_encode", "z2z_lzw_decode", "z2z_step_update", "z2z_lzw_rounds", "z2z_codebook", "z2z_codebook_prefill", "z2z_codebook_usage", "z2z_codebook_prune",
           "z2z_hyper_embed", "z2z_hyper_encode", "z2z_hyper_encode_backward", "z2z_hyper_encode_keep", "z2z_extended_logits", "z2z_extended_logits_static", "z2z_extended_sample", "z2z_extended_nll", "z2z_extended_nll_backward", "z2z_hyper_embed_backward", "z2z_set_option",
           "z2z_read_timing", "z2z_read_launches", "z2z_strerror"]


class Config(ctypes.Structure):
    _fields_ = [("B", c_int32), ("V", c_int32), ("M", c_int32), ("cap", c_int32), ("d", c_int32),
                ("dtype", c_int32), ("pool", c_int32), ("w", c_float * MAX_M)]


class EncoderLayer(ctypes.Structure):
    _fields_ = [(n, c_void_p) for n in ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1",
                                        "b_1", "w_2", "b_2")]


class EncoderDesc(ctypes.Structure):
    _fields_ = [("n_layers", c_int32), ("n_heads", c_int32), ("d_ff", c_int32), ("attention_only", c_int32),
                ("pos", c_void_p), ("layers", ctypes.POINTER(EncoderLayer))]


class Encoder:
    """Device-resident parameters of a learned hyper-encoder, marshalled into the C structs.

    `params`: n_heads, attention_only, d_ff, pos ([M, d] tensor or None) and layers, a list of dicts of
    device tensors named as the fields of z2z_encoder_layer (matrices in the context's dtype, vectors float32).
    The object keeps the tensors alive."""

    def __init__(self, params: dict, torch_dtype):
        self.params = params
        layers = params["layers"]
        self._arr = (EncoderLayer * len(layers))()
        for l, lay in enumerate(layers):
            for name, _ in EncoderLayer._fields_:
                t = lay.get(name)
                if t is None:
                    setattr(self._arr[l], name, None)
                else:
                    setattr(self._arr[l], name, _ptr(t, torch_dtype if name.startswith("w_") else torch.float32))
        self.desc = EncoderDesc()
        self.desc.n_layers = len(layers)
        self.desc.n_heads = int(params["n_heads"])
        self.desc.d_ff = int(params.get("d_ff", 0))
        self.desc.attention_only = 1 if params["attention_only"] else 0
        self.desc.pos = _ptr(params.get("pos"), torch_dtype)
        self.desc.layers = ctypes.cast(self._arr, ctypes.POINTER(EncoderLayer))


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libz2z.so (built in-tree by paper_2506_01084_amd.build); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2506_01084_amd.build` "
                           "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    P32 = POINTER(c_int32)
    lib.z2z_create.argtypes = [POINTER(c_void_p), POINTER(Config)]
    lib.z2z_destroy.argtypes = [c_void_p]
    lib.z2z_reset.argtypes = [c_void_p, c_void_p]
    lib.z2z_lzw_encode.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_int32,
                                   c_void_p, c_void_p]
    lib.z2z_lzw_decode.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_int32,
                                   c_void_p, c_void_p]
    lib.z2z_step_update.argtypes = [c_void_p, c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.z2z_lzw_rounds.argtypes = [c_void_p, POINTER(c_void_p)]
    lib.z2z_codebook.argtypes = [c_void_p, POINTER(c_void_p), POINTER(c_void_p), POINTER(c_void_p)]
    lib.z2z_codebook_prefill.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p,
                                         c_void_p]
    lib.z2z_codebook_usage.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_void_p]
    lib.z2z_codebook_prune.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.z2z_hyper_embed.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_void_p]
    lib.z2z_hyper_encode.argtypes = [c_void_p, c_void_p, POINTER(EncoderDesc), c_void_p, c_void_p, c_int32, c_void_p]
    lib.z2z_hyper_encode_backward.argtypes = [c_void_p, c_void_p, POINTER(EncoderDesc), c_void_p,
                                              POINTER(EncoderDesc), c_void_p, c_int32, c_void_p]
    lib.z2z_hyper_encode_keep.argtypes = [c_void_p, c_void_p, POINTER(EncoderDesc), c_void_p, c_void_p]
    lib.z2z_extended_logits.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                                        c_void_p, c_void_p, c_void_p, c_void_p]
    lib.z2z_extended_logits_static.argtypes = lib.z2z_extended_logits.argtypes
    lib.z2z_extended_sample.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_float, c_int32,
                                        c_float, ctypes.c_uint64, ctypes.c_uint64, c_void_p, c_void_p, c_void_p]
    lib.z2z_extended_nll.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                     c_void_p, c_void_p]
    lib.z2z_extended_nll_backward.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                                              c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.z2z_hyper_embed_backward.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p]
    lib.z2z_set_option.argtypes = [c_void_p, c_int32, c_int32]
    lib.z2z_read_timing.argtypes = [c_void_p, POINTER(c_float), P32]
    lib.z2z_read_launches.argtypes = [c_void_p, POINTER(ctypes.c_int64)]
    lib.z2z_strerror.argtypes = [ctypes.c_int]
    lib.z2z_strerror.restype = c_char_p
    for name in EXPORTS:
        if name != "z2z_strerror":
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


class Z2ZError(RuntimeError):
    pass


def _check(rc: int, what: str) -> None:
    if rc != 0:
        err = Z2ZError(f"{what}: {load_library().z2z_strerror(rc).decode()} ({rc})")
        err.code = rc
        raise err


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Context:
    """One z2z_ctx: B independent sequences sharing V, M, cap, d, dtype and pooling kind."""

    def __init__(self, B: int, V: int, M: int, cap: int, d: int, dtype: str = "bf16", pool: str = "mean",
                 w=None):
        self._lib = load_library()
        cfg = Config()
        cfg.B, cfg.V, cfg.M, cfg.cap, cfg.d = B, V, M, cap, d
        cfg.dtype = {"f32": F32, "bf16": BF16}[dtype]
        cfg.pool = {"mean": POOL_MEAN, "weighted": POOL_WEIGHTED}[pool]
        for j in range(MAX_M):
            cfg.w[j] = float(w[j]) if w is not None and j < len(w) else 0.0
        self.B, self.V, self.M, self.cap, self.d, self.dtype = B, V, M, cap, d, dtype
        self.torch_dtype = torch.float32 if dtype == "f32" else torch.bfloat16
        self._h = c_void_p()
        _check(self._lib.z2z_create(byref(self._h), byref(cfg)), "z2z_create")

    def close(self) -> None:
        if self._h:
            self._lib.z2z_destroy(self._h)
            self._h = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self) -> None:
        _check(self._lib.z2z_reset(self._h, _stream()), "z2z_reset")

    def set_option(self, key: int, value: int) -> None:
        _check(self._lib.z2z_set_option(self._h, key, value), "z2z_set_option")

    def read_timing(self):
        ms, n = c_float(), c_int32()
        _check(self._lib.z2z_read_timing(self._h, byref(ms), byref(n)), "z2z_read_timing")
        return ms.value, n.value

    def read_launches(self) -> dict:
        """Launches enqueued so far per logits kernel family (host-side counters)."""
        arr = (ctypes.c_int64 * 5)()
        _check(self._lib.z2z_read_launches(self._h, arr), "z2z_read_launches")
        return dict(tile_base=arr[0], tile_hyper=arr[1], general=arr[2], decode=arr[3], mid=arr[4])

    # -- the four operations ------------------------------------------------------------------------
    def lzw_encode(self, tokens: torch.Tensor, lens: Optional[torch.Tensor], codes: torch.Tensor,
                   n_codes: torch.Tensor, status: torch.Tensor, flags: int = RESET) -> None:
        assert tokens.shape[0] == self.B and codes.shape[0] == self.B
        _check(self._lib.z2z_lzw_encode(self._h, _ptr(tokens, torch.int32), _ptr(lens, torch.int32),
                                        tokens.shape[1], flags, _ptr(codes, torch.int32),
                                        _ptr(n_codes, torch.int32), codes.shape[1], _ptr(status, torch.int32),
                                        _stream()), "z2z_lzw_encode")

    def lzw_decode(self, codes: torch.Tensor, n_codes: Optional[torch.Tensor], tokens: Optional[torch.Tensor],
                   n_tokens: torch.Tensor, status: torch.Tensor, flags: int = RESET,
                   stride: Optional[int] = None) -> None:
        """`codes` is [B, stride]; with an explicit `stride` it may be any contiguous int32 tensor whose
        element b*stride + i is code i of sequence b (lets a caller point into a larger array)."""
        if stride is None:
            assert codes.shape[0] == self.B
            stride = codes.shape[1]
        out_stride = tokens.shape[1] if tokens is not None else 0
        _check(self._lib.z2z_lzw_decode(self._h, _ptr(codes, torch.int32), _ptr(n_codes, torch.int32),
                                        stride, flags, _ptr(tokens, torch.int32),
                                        _ptr(n_tokens, torch.int32), out_stride, _ptr(status, torch.int32),
                                        _stream()), "z2z_lzw_decode")

    def codebook_prefill(self, phrases: torch.Tensor, phrase_len: torch.Tensor, counts: Optional[torch.Tensor],
                         n_added: torch.Tensor, status: torch.Tensor, flags: int = RESET) -> None:
        assert phrases.dim() == 3 and phrases.shape[0] == self.B and phrases.shape[2] == self.M
        assert tuple(phrase_len.shape) == tuple(phrases.shape[:2])
        _check(self._lib.z2z_codebook_prefill(self._h, _ptr(phrases, torch.int32), _ptr(phrase_len, torch.int32),
                                              _ptr(counts, torch.int32), phrases.shape[1], flags,
                                              _ptr(n_added, torch.int32), _ptr(status, torch.int32), _stream()),
               "z2z_codebook_prefill")

    def codebook_usage(self, codes: torch.Tensor, n_codes: Optional[torch.Tensor], usage: torch.Tensor) -> None:
        assert codes.dim() == 2 and codes.shape[0] == self.B and tuple(usage.shape) == (self.B, self.cap)
        _check(self._lib.z2z_codebook_usage(self._h, _ptr(codes, torch.int32), _ptr(n_codes, torch.int32),
                                            codes.shape[1], _ptr(usage, torch.int32), _stream()), "z2z_codebook_usage")

    def codebook_prune(self, keep: torch.Tensor, new_id: torch.Tensor, n_kept: torch.Tensor) -> None:
        assert tuple(keep.shape) == (self.B, self.cap) and tuple(new_id.shape) == (self.B, self.cap)
        _check(self._lib.z2z_codebook_prune(self._h, _ptr(keep, torch.int32), _ptr(new_id, torch.int32),
                                            _ptr(n_kept, torch.int32), _stream()), "z2z_codebook_prune")

    def step_update(self, codes: torch.Tensor, E: torch.Tensor, W_hyper: torch.Tensor, n_tokens: torch.Tensor,
                    status: torch.Tensor, stride: Optional[int] = None) -> None:
        """One code per sequence (codes[b * stride]) -> codebook update + the newest entry's cache row."""
        if stride is None:
            stride = codes.shape[1] if codes.dim() == 2 else 1
        assert tuple(E.shape) == (self.V, self.d) and tuple(W_hyper.shape) == (self.B, self.cap, self.d)
        _check(self._lib.z2z_step_update(self._h, _ptr(codes, torch.int32), stride, _ptr(E, self.torch_dtype),
                                         _ptr(W_hyper, self.torch_dtype), _ptr(n_tokens, torch.int32),
                                         _ptr(status, torch.int32), _stream()), "z2z_step_update")

    def lzw_rounds(self):
        """Zero-copy int32 [B] device tensor: rounds of the latest parse call per sequence (instrumentation)."""
        r = c_void_p()
        _check(self._lib.z2z_lzw_rounds(self._h, byref(r)), "z2z_lzw_rounds")
        return _device_view(r.value, (self.B,))

    def codebook_ptrs(self):
        e, l, s = c_void_p(), c_void_p(), c_void_p()
        _check(self._lib.z2z_codebook(self._h, byref(e), byref(l), byref(s)), "z2z_codebook")
        return e.value, l.value, s.value

    def codebook(self):
        """Zero-copy int32 device tensors over the borrowed views: entries [B,cap,M], entry_len [B,cap], size [B]."""
        e, l, s = self.codebook_ptrs()
        if self.cap == 0:
            z = torch.empty((self.B, 0, self.M), dtype=torch.int32, device="cuda")
            return z, z[:, :, 0], _device_view(s, (self.B,))
        return (_device_view(e, (self.B, self.cap, self.M)), _device_view(l, (self.B, self.cap)),
                _device_view(s, (self.B,)))

    def hyper_embed(self, E: torch.Tensor, W_hyper: torch.Tensor, first: Optional[torch.Tensor] = None,
                    max_new: int = 0) -> None:
        assert tuple(E.shape) == (self.V, self.d) and tuple(W_hyper.shape) == (self.B, self.cap, self.d)
        _check(self._lib.z2z_hyper_embed(self._h, _ptr(E, self.torch_dtype), _ptr(W_hyper, self.torch_dtype),
                                         _ptr(first, torch.int32), max_new, _stream()), "z2z_hyper_embed")

    def hyper_encode(self, E: torch.Tensor, encoder: "Encoder", W_hyper: torch.Tensor,
                     first: Optional[torch.Tensor] = None, max_new: int = 0) -> None:
        assert tuple(E.shape) == (self.V, self.d) and tuple(W_hyper.shape) == (self.B, self.cap, self.d)
        _check(self._lib.z2z_hyper_encode(self._h, _ptr(E, self.torch_dtype), byref(encoder.desc),
                                          _ptr(W_hyper, self.torch_dtype), _ptr(first, torch.int32), max_new,
                                          _stream()), "z2z_hyper_encode")

    def hyper_encode_keep(self, E: torch.Tensor, encoder: "Encoder", W_hyper: torch.Tensor) -> None:
        assert tuple(E.shape) == (self.V, self.d) and tuple(W_hyper.shape) == (self.B, self.cap, self.d)
        _check(self._lib.z2z_hyper_encode_keep(self._h, _ptr(E, self.torch_dtype), byref(encoder.desc),
                                               _ptr(W_hyper, self.torch_dtype), _stream()), "z2z_hyper_encode_keep")

    def hyper_encode_backward(self, E: torch.Tensor, encoder: "Encoder", dW_hyper: torch.Tensor, grad: "Encoder",
                              dE: torch.Tensor, kept: bool = False) -> None:
        """`grad`: an Encoder built over tensors of the parameters' shapes, which receive the gradients.
        kept=True: use the rows of the preceding hyper_encode_keep call."""
        assert tuple(E.shape) == (self.V, self.d) and tuple(dW_hyper.shape) == (self.B, self.cap, self.d)
        assert tuple(dE.shape) == (self.V, self.d)
        _check(self._lib.z2z_hyper_encode_backward(self._h, _ptr(E, self.torch_dtype), byref(encoder.desc),
                                                   _ptr(dW_hyper, self.torch_dtype), byref(grad.desc),
                                                   _ptr(dE, torch.float32), ENC_KEPT if kept else 0, _stream()),
               "z2z_hyper_encode_backward")

    def _extended_logits(self, fn, what, H, rows_per_seq, W_base, W_hyper, argmax, mx, lse, logits) -> None:
        rows = H.shape[0]
        assert H.shape[1] == self.d and tuple(W_base.shape) == (self.V, self.d)
        assert argmax.numel() == rows and mx.numel() == rows and lse.numel() == rows
        if logits is not None:
            assert tuple(logits.shape) == (rows, self.V + self.cap)
        _check(fn(self._h, _ptr(H, self.torch_dtype), rows, rows_per_seq, _ptr(W_base, self.torch_dtype),
                  _ptr(W_hyper, self.torch_dtype), _ptr(argmax, torch.int32), _ptr(mx, torch.float32),
                  _ptr(lse, torch.float32), _ptr(logits, torch.float32), _stream()), what)

    def extended_logits(self, H: torch.Tensor, rows_per_seq: int, W_base: torch.Tensor, W_hyper: torch.Tensor,
                        argmax: torch.Tensor, mx: torch.Tensor, lse: torch.Tensor,
                        logits: Optional[torch.Tensor] = None) -> None:
        self._extended_logits(self._lib.z2z_extended_logits, "z2z_extended_logits", H, rows_per_seq, W_base, W_hyper,
                              argmax, mx, lse, logits)

    def extended_logits_static(self, H: torch.Tensor, rows_per_seq: int, W_base: torch.Tensor, W_hyper: torch.Tensor,
                               argmax: torch.Tensor, mx: torch.Tensor, lse: torch.Tensor,
                               logits: Optional[torch.Tensor] = None) -> None:
        """The allocation-free entry point: partial reductions in the library's static device array."""
        self._extended_logits(self._lib.z2z_extended_logits_static, "z2z_extended_logits_static", H, rows_per_seq,
                              W_base, W_hyper, argmax, mx, lse, logits)

    def extended_sample(self, H: torch.Tensor, rows_per_seq: int, W_base: torch.Tensor, W_hyper: torch.Tensor,
                        temperature: float, seed: int, step: int, token: torch.Tensor,
                        logprob: Optional[torch.Tensor] = None, top_k: int = 0, top_p: float = 1.0) -> None:
        rows = H.shape[0]
        assert H.shape[1] == self.d and tuple(W_base.shape) == (self.V, self.d)
        assert token.numel() == rows and (logprob is None or logprob.numel() == rows)
        _check(self._lib.z2z_extended_sample(self._h, _ptr(H, self.torch_dtype), rows, rows_per_seq,
                                             _ptr(W_base, self.torch_dtype), _ptr(W_hyper, self.torch_dtype),
                                             float(temperature), int(top_k), float(top_p), int(seed), int(step),
                                             _ptr(token, torch.int32),
                                             _ptr(logprob, torch.float32), _stream()), "z2z_extended_sample")

    def extended_nll(self, H: torch.Tensor, rows_per_seq: int, W_base: torch.Tensor, W_hyper: torch.Tensor,
                     targets: torch.Tensor, nll: torch.Tensor, lse: torch.Tensor) -> None:
        rows = H.shape[0]
        assert H.shape[1] == self.d and tuple(W_base.shape) == (self.V, self.d)
        assert targets.numel() == rows and nll.numel() == rows and lse.numel() == rows
        _check(self._lib.z2z_extended_nll(self._h, _ptr(H, self.torch_dtype), rows, rows_per_seq,
                                          _ptr(W_base, self.torch_dtype), _ptr(W_hyper, self.torch_dtype),
                                          _ptr(targets, torch.int32), _ptr(nll, torch.float32),
                                          _ptr(lse, torch.float32), _stream()), "z2z_extended_nll")

    def extended_nll_backward(self, H: torch.Tensor, rows_per_seq: int, W_base: torch.Tensor, W_hyper: torch.Tensor,
                              targets: torch.Tensor, lse: torch.Tensor, grad_nll: Optional[torch.Tensor],
                              dH: torch.Tensor, dW_base: torch.Tensor, dW_hyper: torch.Tensor) -> None:
        rows = H.shape[0]
        assert H.shape[1] == self.d and tuple(W_base.shape) == (self.V, self.d)
        assert targets.numel() == rows and lse.numel() == rows and (grad_nll is None or grad_nll.numel() == rows)
        assert tuple(dH.shape) == tuple(H.shape) and tuple(dW_base.shape) == tuple(W_base.shape)
        assert tuple(dW_hyper.shape) == (self.B, self.cap, self.d)
        _check(self._lib.z2z_extended_nll_backward(self._h, _ptr(H, self.torch_dtype), rows, rows_per_seq,
                                                   _ptr(W_base, self.torch_dtype), _ptr(W_hyper, self.torch_dtype),
                                                   _ptr(targets, torch.int32), _ptr(lse, torch.float32),
                                                   _ptr(grad_nll, torch.float32), _ptr(dH, self.torch_dtype),
                                                   _ptr(dW_base, self.torch_dtype), _ptr(dW_hyper, self.torch_dtype),
                                                   _stream()), "z2z_extended_nll_backward")

    def hyper_embed_backward(self, dW_hyper: torch.Tensor, dE: torch.Tensor) -> None:
        assert tuple(dW_hyper.shape) == (self.B, self.cap, self.d) and tuple(dE.shape) == (self.V, self.d)
        _check(self._lib.z2z_hyper_embed_backward(self._h, _ptr(dW_hyper, self.torch_dtype), _ptr(dE, torch.float32),
                                                  _stream()), "z2z_hyper_embed_backward")


class _DevView:
    """Describes borrowed int32 device memory through the CUDA array interface (no copy, no ownership)."""

    def __init__(self, ptr: int, shape):
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": "<i4", "data": (int(ptr), False),
                                         "version": 2}


def _device_view(ptr: int, shape) -> torch.Tensor:
    return torch.as_tensor(_DevView(ptr, shape), device="cuda")
