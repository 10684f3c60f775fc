"""Thin ctypes binding of libakvq.so (C ABI in include/akvq.h).

Argument marshalling only: torch supplies device memory and the current stream; every step of the
method runs inside the library's HIP kernels.  There is no fallback: if the library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libakvq.so")

D = 128
MODE_TSA, MODE_PSA, MODE_PSA_SHARED = 0, 1, 2
V_PREROTATED, OUT_ROTATED, K_PREROTATED, Q_PREROTATED, OUT_FP16 = 1, 2, 4, 8, 16

EXPORTS = ["akvq_strerror", "akvq_last_hip_error", "akvq_version", "akvq_cache_bytes",
           "akvq_select_workspace_bytes", "akvq_decode_workspace_bytes", "akvq_decode_default_splits",
           "akvq_decode_split_range",
           "akvq_select_salient", "akvq_quantize_append", "akvq_decode_attention",
           "akvq_quantize_append_tiered", "akvq_decode_attention_tiered", "akvq_quantize_append_rope",
           "akvq_decode_attention_rope", "akvq_decode_step",
           "akvq_decode_static_scratch_bytes", "akvq_decode_attention_static",
           "akvq_massive_workspace_bytes", "akvq_select_massive", "akvq_fold_hadamard", "akvq_stream_read"]
TIER_2BIT, TIER_4BIT_COARSE, TIER_4BIT_FINE, TIER_PAD = 0, 1, 2, 3


class AkvqError(RuntimeError):
    pass


class akvq_window(C.Structure):
    _fields_ = [("k_win", C.c_void_p), ("v_win", C.c_void_p), ("W", C.c_int32)]


class akvq_rope(C.Structure):
    _fields_ = [("cos", C.c_void_p), ("sin", C.c_void_p), ("batch_stride", C.c_int64)]


class akvq_cache(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hkv", C.c_int32), ("G", C.c_int32), ("T_cap", C.c_int32),
                ("S_cap", C.c_int32), ("T_len", C.c_int32),
                ("k_codes", C.c_void_p), ("v_codes", C.c_void_p), ("k_meta", C.c_void_p), ("v_meta", C.c_void_p),
                ("k_sal", C.c_void_p), ("v_sal", C.c_void_p), ("sal_idx", C.c_void_p), ("sal_cnt", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Load the library built by paper_2501_15021_amd.build (never builds, never falls back)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise AkvqError(f"{LIB_PATH} is missing: run `python -m paper_2501_15021_amd.build` "
                            "(or __graft_entry__.build()) first; there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        L.akvq_strerror.restype = C.c_char_p
        L.akvq_strerror.argtypes = [C.c_int]
        L.akvq_last_hip_error.restype = C.c_int
        L.akvq_version.restype = C.c_int
        L.akvq_cache_bytes.restype = C.c_int
        L.akvq_cache_bytes.argtypes = [C.POINTER(akvq_cache), C.POINTER(C.c_size_t)]
        L.akvq_select_workspace_bytes.restype = C.c_size_t
        L.akvq_select_workspace_bytes.argtypes = [C.c_int] * 5
        L.akvq_decode_workspace_bytes.restype = C.c_size_t
        L.akvq_decode_workspace_bytes.argtypes = [C.c_int] * 3
        L.akvq_decode_default_splits.restype = C.c_int
        L.akvq_decode_default_splits.argtypes = [C.c_int] * 3
        L.akvq_decode_split_range.restype = C.c_int
        L.akvq_decode_split_range.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.akvq_select_salient.restype = C.c_int
        L.akvq_select_salient.argtypes = [C.POINTER(akvq_cache), C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                          C.c_int, C.c_int, C.c_int, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t,
                                          C.c_void_p]
        L.akvq_quantize_append.restype = C.c_int
        L.akvq_quantize_append.argtypes = [C.POINTER(akvq_cache), C.c_void_p, C.c_void_p, C.c_int, C.c_float,
                                           C.c_uint32, C.c_void_p]
        L.akvq_decode_attention.restype = C.c_int
        L.akvq_decode_attention.argtypes = [C.POINTER(akvq_cache), C.c_void_p, C.c_int, C.c_float, C.c_void_p,
                                            C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p]
        L.akvq_decode_static_scratch_bytes.restype = C.c_size_t
        L.akvq_decode_static_scratch_bytes.argtypes = []
        L.akvq_decode_attention_static.restype = C.c_int
        L.akvq_decode_attention_static.argtypes = [C.POINTER(akvq_cache), C.c_void_p, C.c_int, C.c_float, C.c_void_p,
                                                   C.c_void_p, C.c_int, C.c_uint32, C.c_void_p]
        L.akvq_stream_read.restype = C.c_int
        L.akvq_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_int, C.c_void_p]
        L.akvq_fold_hadamard.restype = C.c_int
        L.akvq_fold_hadamard.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.akvq_massive_workspace_bytes.restype = C.c_size_t
        L.akvq_massive_workspace_bytes.argtypes = [C.c_int, C.c_int]
        L.akvq_select_massive.restype = C.c_int
        L.akvq_select_massive.argtypes = [C.POINTER(akvq_cache), C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float,
                                          C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.akvq_quantize_append_tiered.restype = C.c_int
        L.akvq_quantize_append_tiered.argtypes = [C.POINTER(akvq_cache), C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                                  C.c_void_p, C.c_int, C.c_float, C.c_float, C.c_void_p,
                                                  C.POINTER(akvq_window), C.c_uint32, C.c_void_p]
        L.akvq_decode_attention_tiered.restype = C.c_int
        L.akvq_decode_attention_tiered.argtypes = [C.POINTER(akvq_cache), C.c_void_p, C.POINTER(akvq_window),
                                                   C.c_void_p, C.c_int, C.c_float, C.c_void_p, C.c_void_p, C.c_int,
                                                   C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p]
        L.akvq_quantize_append_rope.restype = C.c_int
        L.akvq_quantize_append_rope.argtypes = [C.POINTER(akvq_cache), C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                                C.c_void_p, C.c_int, C.c_float, C.c_float, C.c_void_p,
                                                C.POINTER(akvq_window), C.POINTER(akvq_rope), C.c_uint32, C.c_void_p]
        L.akvq_decode_attention_rope.restype = C.c_int
        L.akvq_decode_attention_rope.argtypes = [C.POINTER(akvq_cache), C.c_void_p, C.POINTER(akvq_window), C.c_void_p,
                                                 C.POINTER(akvq_rope), C.c_int, C.c_float, C.c_void_p, C.c_void_p,
                                                 C.c_int, C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p]
        L.akvq_decode_step.restype = C.c_int
        L.akvq_decode_step.argtypes = [C.POINTER(akvq_cache), C.c_void_p, C.POINTER(akvq_window), C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.POINTER(akvq_rope), C.c_int, C.c_float, C.c_float, C.c_void_p,
                                       C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p]
        _lib = L
    return _lib


def _rope_struct(rope, B: int, n: int):
    """(cos, sin) fp16 tensors [n, 64] (one table for the batch) or [B, n, 64] -> akvq_rope (tensors stay referenced)."""
    cos, sin = rope
    assert cos.dtype == torch.float16 and sin.dtype == torch.float16 and cos.is_contiguous() and sin.is_contiguous()
    assert cos.shape == sin.shape and tuple(cos.shape[-2:]) == (n, 64)
    assert cos.dim() == 2 or (cos.dim() == 3 and cos.shape[0] == B)
    return akvq_rope(cos.data_ptr(), sin.data_ptr(), n * 64 if cos.dim() == 3 else 0)


def _check(status: int, what: str):
    if status != 0:
        L = lib()
        raise AkvqError(f"{what}: {L.akvq_strerror(status).decode()} (status {status}, hip {L.akvq_last_hip_error()})")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Cache:
    """One layer's mixed-precision cache: device tensors plus the plain-C descriptor the library takes."""

    def __init__(self, B: int, Hkv: int, G: int, T_cap: int, S_cap: int, device="cuda", fill: Optional[int] = None):
        self.B, self.Hkv, self.G, self.T_cap, self.S_cap, self.T_len = B, Hkv, G, T_cap, S_cap, 0
        self.fine_mask: Optional[torch.Tensor] = None  # [B, T_cap/32] int32, created by the first tiered append
        self.W = 0                                     # recent-window length (enable_window)
        self.k_win: Optional[torch.Tensor] = None      # [B, Hkv, W, 128] bf16 bits, ring by row % W
        self.v_win: Optional[torch.Tensor] = None      # [B, Hkv, W/32, 4096] bf16 bits, tiled
        shape = akvq_cache(B, Hkv, G, T_cap, S_cap, 0)
        sizes = (C.c_size_t * 8)()
        _check(lib().akvq_cache_bytes(C.byref(shape), sizes), "akvq_cache_bytes")
        dev = torch.device(device)
        mk = (lambda n: torch.empty(n, dtype=torch.uint8, device=dev)) if fill is None else \
             (lambda n: torch.full((n,), fill, dtype=torch.uint8, device=dev))
        self.k_codes = mk(sizes[0]).view(torch.int32).view(B, Hkv, T_cap // 32, 256)
        self.v_codes = mk(sizes[1]).view(torch.int32).view(B, Hkv, T_cap // 32, 256)
        self.k_meta = mk(sizes[2]).view(torch.int32).view(B, Hkv, T_cap, D // G)
        self.v_meta = mk(sizes[3]).view(torch.int32).view(B, Hkv, T_cap, D // G)
        # the overlay is zero-filled: decode masks unused slots, zeroing keeps them finite for other readers
        self.k_sal = torch.zeros(sizes[4] // 2, dtype=torch.int16, device=dev).view(B, Hkv, S_cap, D)
        self.v_sal = torch.zeros(sizes[5] // 2, dtype=torch.int16, device=dev).view(B, Hkv, S_cap // 32, 4096)
        self.sal_idx = torch.full((B, Hkv, S_cap), -1, dtype=torch.int32, device=dev)
        self.sal_cnt = torch.zeros(sizes[7] // 4, dtype=torch.int32, device=dev)
        self._ws = {}

    def struct(self) -> akvq_cache:
        return akvq_cache(self.B, self.Hkv, self.G, self.T_cap, self.S_cap, self.T_len,
                          self.k_codes.data_ptr(), self.v_codes.data_ptr(), self.k_meta.data_ptr(),
                          self.v_meta.data_ptr(), self.k_sal.data_ptr(), self.v_sal.data_ptr(),
                          self.sal_idx.data_ptr(), self.sal_cnt.data_ptr())

    def workspace(self, key: str, nbytes: int) -> torch.Tensor:
        ws = self._ws.get(key)
        if ws is None or ws.numel() < nbytes:
            ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.k_codes.device)
            self._ws[key] = ws
        return ws

    def enable_window(self, W: int):
        """Keep the most recent W rows 16-bit (zero-initialised rings)."""
        assert W > 0 and W % 64 == 0
        dev = self.k_codes.device
        self.W = W
        self.k_win = torch.zeros(self.B, self.Hkv, W, D, dtype=torch.int16, device=dev)
        self.v_win = torch.zeros(self.B, self.Hkv, W // 32, 4096, dtype=torch.int16, device=dev)

    def window_struct(self):
        if self.W == 0:
            return None
        return akvq_window(self.k_win.data_ptr(), self.v_win.data_ptr(), self.W)

    def counts(self) -> torch.Tensor:
        return self.sal_cnt[: self.B * self.Hkv].view(self.B, self.Hkv)

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in (self.k_codes, self.v_codes, self.k_meta, self.v_meta,
                                                          self.k_sal, self.v_sal, self.sal_idx, self.sal_cnt))


def select_salient(cache: Cache, mode: int, *, is_text: Optional[torch.Tensor] = None,
                   q_tail: Optional[torch.Tensor] = None, k: Optional[torch.Tensor] = None, top_k: int = 0,
                   sm_scale: float = 0.0, mass_out: Optional[torch.Tensor] = None) -> None:
    """akvq_select_salient: writes cache.sal_idx / cache.sal_cnt on the current stream."""
    c = cache.struct()
    if mode == MODE_TSA:
        assert is_text.dtype == torch.uint8 and is_text.is_contiguous() and is_text.shape[0] == cache.B
        st = lib().akvq_select_salient(C.byref(c), mode, _ptr(is_text), None, cache.Hkv, None, is_text.shape[1], 0, 0,
                                       0.0, None, None, 0, _stream())
    else:
        assert q_tail.dtype == torch.float16 and k.dtype == torch.float16
        assert q_tail.is_contiguous() and k.is_contiguous()
        B, Hq, W, _ = q_tail.shape
        T = k.shape[2]
        nws = lib().akvq_select_workspace_bytes(B, Hq, cache.Hkv, T, W)
        ws = cache.workspace("select", nws)
        if mass_out is not None:
            assert mass_out.dtype == torch.float32 and mass_out.is_contiguous()
        st = lib().akvq_select_salient(C.byref(c), mode, None, _ptr(q_tail), Hq, _ptr(k), T, W, top_k, sm_scale,
                                       _ptr(mass_out), _ptr(ws), ws.numel(), _stream())
    _check(st, "akvq_select_salient")


def fold_hadamard(w: torch.Tensor, axis: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """akvq_fold_hadamard: fold H_128 into a projection matrix [rows, cols] fp16 (axis 1: W_V, axis 0: W_O)."""
    assert w.dtype == torch.float16 and w.is_contiguous() and w.dim() == 2
    if out is None:
        out = torch.empty_like(w)
    assert out.dtype == torch.float16 and out.is_contiguous() and out.shape == w.shape
    _check(lib().akvq_fold_hadamard(_ptr(w), _ptr(out), w.shape[0], w.shape[1], axis, _stream()), "akvq_fold_hadamard")
    return out


def stream_read(src: torch.Tensor, sink: torch.Tensor, non_temporal: bool = True) -> None:
    """akvq_stream_read: one plain 128-bit streaming-read pass over src (measurement aid)."""
    assert src.is_contiguous() and sink.dtype == torch.int32 and sink.numel() >= 1
    _check(lib().akvq_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), int(non_temporal), _stream()),
           "akvq_stream_read")


def select_massive(cache: Cache, hidden: torch.Tensor, top_k: int, floor: float = 0.0,
                   score_out: Optional[torch.Tensor] = None) -> None:
    """akvq_select_massive: pivots = top_k tokens by largest hidden-state magnitude (>= floor); hidden [B,T,d_model]."""
    assert hidden.dtype == torch.float16 and hidden.is_contiguous()
    B, T, d_model = hidden.shape
    ws = cache.workspace("massive", lib().akvq_massive_workspace_bytes(B, T))
    c = cache.struct()
    _check(lib().akvq_select_massive(C.byref(c), _ptr(hidden), T, d_model, top_k, floor, _ptr(score_out), _ptr(ws),
                                     ws.numel(), _stream()), "akvq_select_massive")


def quantize_append(cache: Cache, k_new: torch.Tensor, v_new: torch.Tensor, clip: float, flags: int = 0) -> None:
    """akvq_quantize_append for rows [T_len, T_len + n_new); advances cache.T_len."""
    assert k_new.dtype == torch.float16 and v_new.dtype == torch.float16
    assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.shape == v_new.shape
    n_new = k_new.shape[2]
    c = cache.struct()
    _check(lib().akvq_quantize_append(C.byref(c), _ptr(k_new), _ptr(v_new), n_new, clip, flags, _stream()),
           "akvq_quantize_append")
    cache.T_len += n_new


def quantize_append_tiered(cache: Cache, k_src: torch.Tensor, v_src: torch.Tensor, row_src: torch.Tensor,
                           row_tier: torch.Tensor, clip2: float, clip4: float, flags: int = 0, rope=None) -> None:
    """akvq_quantize_append_tiered: cache rows [T_len, T_len + n_rows) from source tokens row_src [B, n_rows] int32
    with tiers row_tier [B, n_rows] uint8; keeps the fine-half mask in cache.fine_mask; advances cache.T_len.
    rope = (cos, sin): k_src holds pre-RoPE rows (akvq_quantize_append_rope)."""
    assert k_src.dtype == torch.float16 and v_src.dtype == torch.float16
    assert k_src.is_contiguous() and v_src.is_contiguous() and k_src.shape == v_src.shape
    n_src = k_src.shape[2]
    if row_src is None:      # plain rows, identity mapping (what differs from quantize_append is the window)
        assert row_tier is None
        n_rows, mask = n_src, None
    else:
        assert row_src.dtype == torch.int32 and row_tier.dtype == torch.uint8
        assert row_src.is_contiguous() and row_tier.is_contiguous() and row_src.shape == row_tier.shape
        n_rows = row_src.shape[1]
        if cache.fine_mask is None:
            cache.fine_mask = torch.zeros(cache.B, cache.T_cap // 32, dtype=torch.int32, device=k_src.device)
        mask = cache.fine_mask
    c = cache.struct()
    win = cache.window_struct()
    if rope is not None:
        rs = _rope_struct(rope, cache.B, n_src)
        _check(lib().akvq_quantize_append_rope(C.byref(c), _ptr(k_src), _ptr(v_src), n_src, _ptr(row_src),
                                               _ptr(row_tier), n_rows, clip2, clip4, _ptr(mask),
                                               C.byref(win) if win else None, C.byref(rs), flags, _stream()),
               "akvq_quantize_append_rope")
    else:
        _check(lib().akvq_quantize_append_tiered(C.byref(c), _ptr(k_src), _ptr(v_src), n_src, _ptr(row_src),
                                                 _ptr(row_tier), n_rows, clip2, clip4, _ptr(mask),
                                                 C.byref(win) if win else None, flags, _stream()),
               "akvq_quantize_append_tiered")
    cache.T_len += n_rows


def decode_attention(cache: Cache, q: torch.Tensor, sm_scale: float, n_split: int = 0, flags: int = 0,
                     out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None, rope=None):
    """akvq_decode_attention: returns (out [B,Hq,128] fp32, lse [B,Hq] fp32).
    rope = (cos, sin) [1, 64] or [B, 1, 64]: q holds pre-RoPE queries (akvq_decode_attention_rope)."""
    assert q.dtype == torch.float16 and q.is_contiguous()
    B, Hq, _ = q.shape
    if n_split <= 0:
        n_split = lib().akvq_decode_default_splits(cache.B, cache.Hkv, cache.T_len)
    ws = cache.workspace("decode", lib().akvq_decode_workspace_bytes(B, Hq, n_split))
    out_dtype = torch.float16 if flags & OUT_FP16 else torch.float32
    if out is None:
        out = torch.empty(B, Hq, D, dtype=out_dtype, device=q.device)
    assert out.dtype == out_dtype and out.is_contiguous()
    if lse is None:
        lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    c = cache.struct()
    if rope is not None:
        win = cache.window_struct()
        rs = _rope_struct(rope, B, 1)
        _check(lib().akvq_decode_attention_rope(C.byref(c), _ptr(cache.fine_mask), C.byref(win) if win else None,
                                                _ptr(q), C.byref(rs), Hq, sm_scale, _ptr(out), _ptr(lse), n_split,
                                                _ptr(ws), ws.numel(), flags, _stream()), "akvq_decode_attention_rope")
        return out, lse
    if cache.fine_mask is not None or cache.W:
        win = cache.window_struct()
        _check(lib().akvq_decode_attention_tiered(C.byref(c), _ptr(cache.fine_mask), C.byref(win) if win else None,
                                                  _ptr(q), Hq, sm_scale, _ptr(out), _ptr(lse), n_split, _ptr(ws),
                                                  ws.numel(), flags, _stream()), "akvq_decode_attention_tiered")
        return out, lse
    _check(lib().akvq_decode_attention(C.byref(c), _ptr(q), Hq, sm_scale, _ptr(out), _ptr(lse), n_split, _ptr(ws),
                                       ws.numel(), flags, _stream()), "akvq_decode_attention")
    return out, lse


def decode_attention_static(cache: Cache, q: torch.Tensor, sm_scale: float, out: torch.Tensor, lse: torch.Tensor,
                            n_split: int = 0, flags: int = 0) -> None:
    """akvq_decode_attention_static: the partials live in the library's fixed device array; the caller supplies out
    [B,Hq,128] fp32 and lse [B,Hq] fp32, and nothing is allocated on the way."""
    assert q.dtype == torch.float16 and q.is_contiguous()
    assert out.dtype == torch.float32 and out.is_contiguous() and lse.dtype == torch.float32 and lse.is_contiguous()
    B, Hq, _ = q.shape
    assert tuple(out.shape) == (B, Hq, D) and tuple(lse.shape) == (B, Hq)
    c = cache.struct()
    _check(lib().akvq_decode_attention_static(C.byref(c), _ptr(q), Hq, sm_scale, _ptr(out), _ptr(lse), n_split, flags,
                                              _stream()), "akvq_decode_attention_static")


def decode_step(cache: Cache, k_new: torch.Tensor, v_new: torch.Tensor, q: torch.Tensor, clip: float, sm_scale: float,
                n_split: int = 0, flags: int = 0, out: Optional[torch.Tensor] = None,
                lse: Optional[torch.Tensor] = None, rope=None):
    """akvq_decode_step: append one row per (batch, kv-head) and run decode attention over the cache including it, in
    one launch; advances cache.T_len.  Returns (out, lse)."""
    assert k_new.dtype == torch.float16 and v_new.dtype == torch.float16 and q.dtype == torch.float16
    assert k_new.is_contiguous() and v_new.is_contiguous() and q.is_contiguous()
    assert tuple(k_new.shape) == (cache.B, cache.Hkv, 1, D) and k_new.shape == v_new.shape
    B, Hq, _ = q.shape
    if n_split <= 0:
        n_split = lib().akvq_decode_default_splits(cache.B, cache.Hkv, cache.T_len + 1)
    ws = cache.workspace("decode", lib().akvq_decode_workspace_bytes(B, Hq, n_split))
    if out is None:
        out = torch.empty(B, Hq, D, dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    c = cache.struct()
    win = cache.window_struct()
    rs = _rope_struct(rope, B, 1) if rope is not None else None
    _check(lib().akvq_decode_step(C.byref(c), _ptr(cache.fine_mask), C.byref(win) if win else None, _ptr(k_new),
                                  _ptr(v_new), _ptr(q), C.byref(rs) if rs is not None else None, Hq, clip, sm_scale,
                                  _ptr(out), _ptr(lse), n_split, _ptr(ws), ws.numel(), flags, _stream()),
           "akvq_decode_step")
    cache.T_len += 1
    return out, lse
