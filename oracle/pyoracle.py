"""ctypes/numpy front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this module.
It never touches the GPU library.  All arrays are host numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libakvq_oracle.so")
_SRC = os.path.join(_HERE, "akvq_oracle.c")

D = 128


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
               "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


class _Cache(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hkv", C.c_int32), ("G", C.c_int32), ("T_cap", C.c_int32),
                ("S_cap", C.c_int32), ("T_len", C.c_int32),
                ("k_codes", C.c_void_p), ("v_codes", C.c_void_p), ("k_meta", C.c_void_p), ("v_meta", C.c_void_p),
                ("k_sal", C.c_void_p), ("v_sal", C.c_void_p), ("sal_idx", C.c_void_p), ("sal_cnt", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_SO)
        L.orc_half_to_float.restype = C.c_float
        L.orc_half_to_float.argtypes = [C.c_uint16]
        L.orc_float_to_half_rne.restype = C.c_uint16
        L.orc_float_to_half_rne.argtypes = [C.c_float]
        L.orc_bf16_to_float.restype = C.c_float
        L.orc_bf16_to_float.argtypes = [C.c_uint16]
        L.orc_float_to_bf16_rne.restype = C.c_uint16
        L.orc_float_to_bf16_rne.argtypes = [C.c_float]
        L.orc_hadamard_dense.argtypes = [C.c_int, C.c_void_p]
        L.orc_wht_dense_f64.argtypes = [C.c_int, C.c_void_p, C.c_void_p]
        L.orc_fwht128_f32.argtypes = [C.c_void_p, C.c_void_p]
        L.orc_quantize_row.argtypes = [C.c_void_p, C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p]
        L.orc_dequant.restype = C.c_double
        L.orc_dequant.argtypes = [C.c_uint8, C.c_uint16, C.c_int16]
        L.orc_k_code_pos.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_size_t), C.POINTER(C.c_int)]
        L.orc_v_code_pos.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_size_t), C.POINTER(C.c_int)]
        L.orc_vsal_pos.restype = C.c_size_t
        L.orc_vsal_pos.argtypes = [C.c_int, C.c_int]
        L.orc_get_code.restype = C.c_uint8
        L.orc_get_code.argtypes = [C.POINTER(_Cache), C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_select_tsa.argtypes = [C.POINTER(_Cache), C.c_void_p, C.c_int]
        L.orc_select_psa.argtypes = [C.POINTER(_Cache), C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                     C.c_double, C.c_void_p]
        L.orc_select_psa_shared.argtypes = L.orc_select_psa.argtypes
        L.orc_quantize_append.argtypes = [C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_int]
        L.orc_decode_attention.argtypes = [C.POINTER(_Cache), C.c_int, C.c_void_p, C.c_double, C.c_int, C.c_void_p,
                                           C.c_void_p]
        L.orc_decode_attention_one.argtypes = [C.POINTER(_Cache), C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_double,
                                               C.c_int, C.c_void_p, C.c_void_p]
        L.orc_fold_hadamard.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int]
        L.orc_select_massive.argtypes = [C.POINTER(_Cache), C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float,
                                         C.c_void_p]
        L.orc_quantize_row_bits.argtypes = [C.c_void_p, C.c_int, C.c_float, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p]
        L.orc_quantize_append_tiered.argtypes = [C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                                 C.c_void_p, C.c_int, C.c_float, C.c_float, C.c_int, C.c_void_p,
                                                 C.c_void_p, C.c_void_p, C.c_int]
        L.orc_decode_attention_tiered.argtypes = [C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                                  C.c_int, C.c_void_p, C.c_double, C.c_int, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _p(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a) -> np.ndarray:
    """fp16 numpy array (or uint16 bit patterns) -> contiguous uint16 bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


@dataclass
class OracleCache:
    """Host mirror of one layer's cache, in the documented byte format."""
    B: int
    Hkv: int
    G: int
    T_cap: int
    S_cap: int
    T_len: int = 0
    fill: int = 0  # byte value used to initialise the planes (tests use a non-zero one to show RMW is clean)
    k_codes: np.ndarray = field(init=False)
    v_codes: np.ndarray = field(init=False)
    k_meta: np.ndarray = field(init=False)
    v_meta: np.ndarray = field(init=False)
    k_sal: np.ndarray = field(init=False)
    v_sal: np.ndarray = field(init=False)
    sal_idx: np.ndarray = field(init=False)
    sal_cnt: np.ndarray = field(init=False)
    fine_mask: np.ndarray | None = field(init=False, default=None)  # [B, T_cap/32] uint32, set by the tiered append
    W: int = field(init=False, default=0)                           # recent-window length (0 = none)
    k_win: np.ndarray | None = field(init=False, default=None)      # [B, Hkv, W, 128] bf16 bits, ring by t % W
    v_win: np.ndarray | None = field(init=False, default=None)      # [B, Hkv, W/32, 4096] bf16 bits, tiled

    def __post_init__(self):
        assert self.T_cap % 64 == 0 and self.S_cap % 64 == 0 and self.G in (64, 128)
        B, H, ng = self.B, self.Hkv, D // self.G
        f32 = np.uint32(self.fill * 0x01010101)
        self.k_codes = np.full((B, H, self.T_cap // 32, 256), f32, dtype=np.uint32)
        self.v_codes = np.full((B, H, self.T_cap // 32, 256), f32, dtype=np.uint32)
        self.k_meta = np.full((B, H, self.T_cap, ng), f32, dtype=np.uint32)
        self.v_meta = np.full((B, H, self.T_cap, ng), f32, dtype=np.uint32)
        self.k_sal = np.zeros((B, H, self.S_cap, D), dtype=np.uint16)
        self.v_sal = np.zeros((B, H, self.S_cap // 32, 4096), dtype=np.uint16)
        self.sal_idx = np.full((B, H, self.S_cap), -1, dtype=np.int32)
        self.sal_cnt = np.zeros((B, H), dtype=np.int32)

    def _c(self) -> _Cache:
        return _Cache(self.B, self.Hkv, self.G, self.T_cap, self.S_cap, self.T_len,
                      _p(self.k_codes), _p(self.v_codes), _p(self.k_meta), _p(self.v_meta),
                      _p(self.k_sal), _p(self.v_sal), _p(self.sal_idx), _p(self.sal_cnt))

    # ---- the three calls ----
    def select_tsa(self, is_text: np.ndarray):
        is_text = np.ascontiguousarray(is_text, dtype=np.uint8)
        assert is_text.shape[0] == self.B
        c = self._c()
        lib().orc_select_tsa(C.byref(c), _p(is_text), is_text.shape[1])

    def select_psa(self, q_tail, k, top_k: int, sm_scale: float, want_mass: bool = False, share_heads: bool = False):
        q_tail, k = _u16(q_tail), _u16(k)
        B, Hq, W, _ = q_tail.shape
        T = k.shape[2]
        assert k.shape[:2] == (self.B, self.Hkv) and B == self.B
        mass = np.zeros((self.B, self.Hkv, T), dtype=np.float64) if want_mass else None
        c = self._c()
        fn = lib().orc_select_psa_shared if share_heads else lib().orc_select_psa
        fn(C.byref(c), Hq, _p(q_tail), _p(k), T, W, top_k, sm_scale, _p(mass))
        return mass

    def quantize_append(self, k_new, v_new, clip: float, rotate_v: bool = True, rotate_k: bool = True):
        k_new, v_new = _u16(k_new), _u16(v_new)
        n_new = k_new.shape[2]
        assert k_new.shape == (self.B, self.Hkv, n_new, D) == v_new.shape
        assert self.T_len + n_new <= self.T_cap
        c = self._c()
        lib().orc_quantize_append(C.byref(c), _p(k_new), _p(v_new), n_new, clip, int(rotate_k) + 2 * int(rotate_v))
        self.T_len += n_new

    def select_massive(self, hidden, top_k: int, floor: float = 0.0, want_score: bool = False):
        """Pivots = top_k tokens by largest hidden-state magnitude (>= floor); hidden [B, T, d_model] fp16."""
        hidden = _u16(hidden)
        B, T, d_model = hidden.shape
        assert B == self.B
        score = np.zeros((B, T), dtype=np.float64) if want_score else None
        c = self._c()
        lib().orc_select_massive(C.byref(c), _p(hidden), T, d_model, top_k, floor, _p(score))
        return score

    def enable_window(self, W: int):
        """Keep the most recent W rows 16-bit (ring buffers, zero-initialised)."""
        assert W % 64 == 0 and W > 0
        self.W = W
        self.k_win = np.zeros((self.B, self.Hkv, W, D), dtype=np.uint16)
        self.v_win = np.zeros((self.B, self.Hkv, W // 32, 4096), dtype=np.uint16)

    def quantize_append_tiered(self, k_src, v_src, row_src, row_tier, clip2: float, clip4: float,
                               rotate_v: bool = True, rotate_k: bool = True):
        """Rows [T_len, T_len + n_rows): row r of batch b takes source token row_src[b, r] with tier row_tier[b, r]
        (0 = 2-bit, 1 / 2 = coarse / fine half of a 4-bit token, 3 = padding); updates self.fine_mask."""
        k_src, v_src = _u16(k_src), _u16(v_src)
        n_src = k_src.shape[2]
        if row_src is None:      # plain rows, identity mapping (only the window differs from quantize_append)
            n_rows = n_src
            assert row_tier is None
        else:
            row_src = np.ascontiguousarray(row_src, dtype=np.int32)
            row_tier = np.ascontiguousarray(row_tier, dtype=np.uint8)
            n_rows = row_src.shape[1]
            assert row_src.shape == (self.B, n_rows) == row_tier.shape
            if self.fine_mask is None:
                self.fine_mask = np.zeros((self.B, self.T_cap // 32), dtype=np.uint32)
        assert k_src.shape == (self.B, self.Hkv, n_src, D) == v_src.shape
        assert self.T_len + n_rows <= self.T_cap
        c = self._c()
        lib().orc_quantize_append_tiered(C.byref(c), _p(k_src), _p(v_src), n_src, _p(row_src), _p(row_tier), n_rows,
                                         clip2, clip4, int(rotate_k) + 2 * int(rotate_v), _p(self.fine_mask if row_src is not None else None),
                                         _p(self.k_win), _p(self.v_win), self.W)
        self.T_len += n_rows

    def decode(self, q, sm_scale: float, unrotate: bool = True, rotate_q: bool = True):
        q = _u16(q)
        B, Hq, _ = q.shape
        out = np.zeros((B, Hq, D), dtype=np.float64)
        lse = np.zeros((B, Hq), dtype=np.float64)
        c = self._c()
        lib().orc_decode_attention_tiered(C.byref(c), _p(self.fine_mask), _p(self.k_win), _p(self.v_win), self.W, Hq,
                                          _p(q), sm_scale, int(rotate_q) + 2 * int(unrotate), _p(out), _p(lse))
        return out, lse

    def decode_one(self, b: int, hq: int, Hq: int, q_row, sm_scale: float, unrotate: bool = True,
                   rotate_q: bool = True):
        q_row = _u16(q_row)
        out = np.zeros(D, dtype=np.float64)
        lse = np.zeros(1, dtype=np.float64)
        c = self._c()
        lib().orc_decode_attention_one(C.byref(c), Hq, b, hq, _p(q_row), sm_scale, int(rotate_q) + 2 * int(unrotate), _p(out), _p(lse))
        return out, float(lse[0])

    def get_code(self, tensor: int, b: int, h: int, t: int, e: int) -> int:
        c = self._c()
        return int(lib().orc_get_code(C.byref(c), tensor, b, h, t, e))


# ---- thin wrappers of the row-level functions ----
def hadamard_dense(n: int) -> np.ndarray:
    H = np.zeros((n, n), dtype=np.float64)
    lib().orc_hadamard_dense(n, _p(H))
    return H


def wht_dense(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.zeros_like(x)
    lib().orc_wht_dense_f64(x.shape[-1], _p(x), _p(y))
    return y


def fwht128_f32(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.shape == (D,)
    u = np.zeros_like(x)
    lib().orc_fwht128_f32(_p(x), _p(u))
    return u


def quantize_row(x_f16, G: int, clip: float, rotate: bool = True):
    x = _u16(x_f16)
    assert x.shape == (D,)
    codes = np.zeros(D, dtype=np.uint8)
    sb = np.zeros(D // G, dtype=np.uint16)
    z = np.zeros(D // G, dtype=np.int16)
    ybf = np.zeros(D, dtype=np.uint16)
    lib().orc_quantize_row(_p(x), G, clip, int(rotate), _p(codes), _p(sb), _p(z), _p(ybf))
    return codes, sb, z, ybf


def quantize_row_bits(x_f16, G: int, clip: float, n_bits: int, rotate: bool = True):
    x = _u16(x_f16)
    assert x.shape == (D,)
    codes = np.zeros(D, dtype=np.uint8)
    sb = np.zeros(D // G, dtype=np.uint16)
    z = np.zeros(D // G, dtype=np.int16)
    ybf = np.zeros(D, dtype=np.uint16)
    lib().orc_quantize_row_bits(_p(x), G, clip, int(rotate), n_bits, _p(codes), _p(sb), _p(z), _p(ybf))
    return codes, sb, z, ybf


def fold_hadamard(w_f16, axis: int) -> np.ndarray:
    """Fold H_128 into a projection matrix [rows, cols] fp16 (axis 1: column runs of every row; axis 0: row runs)."""
    w = _u16(w_f16)
    rows, cols = w.shape
    assert (cols if axis == 1 else rows) % D == 0
    out = np.zeros_like(w)
    lib().orc_fold_hadamard(_p(w), _p(out), rows, cols, axis)
    return out.view(np.float16)


def rope_rows(x_f16, cos_f16, sin_f16) -> np.ndarray:
    """Rotary position embedding (channel i pairs with i + 64) of x [B, H, n, 128] fp16 with fp16 tables cos, sin
    [n, 64] (shared) or [B, n, 64]; rounded to fp16.  Applied to pre-RoPE K before the write path / q before decode."""
    x = _u16(x_f16)
    B, H, n, d = x.shape
    assert d == D
    cos, sin = _u16(cos_f16), _u16(sin_f16)
    assert cos.shape == sin.shape and cos.shape[-2:] == (n, 64)
    stride = n * 64 if cos.ndim == 3 else 0
    assert cos.ndim == 2 or cos.shape[0] == B
    out = np.zeros_like(x)
    lib().orc_rope_rows(_p(x), _p(out), B, H, n, _p(cos), _p(sin), C.c_long(stride))
    return out.view(np.float16)


def topk_margins(mass: np.ndarray, top_k: int) -> np.ndarray:
    """Relative gap at the selection boundary of each row of fp64 masses [..., T]: (m_k - m_{k+1}) / m_k with
    m_1 >= m_2 >= ... the row sorted descending.  A top-k set is unique, and reproducible by an implementation whose
    masses carry a relative error well below this gap, only when the gap is large enough; inputs for exact index-set
    comparison are accepted on it.  inf when the row has no (k+1)-th element; 0 when m_k is 0 (a tie among zeros)."""
    mass = np.asarray(mass, dtype=np.float64)
    T = mass.shape[-1]
    if top_k >= T:
        return np.full(mass.shape[:-1], np.inf)
    top = -np.partition(-mass, top_k, axis=-1)[..., :top_k + 1]      # the k+1 largest, the (k+1)-th in place
    m_k, m_next = top[..., :top_k].min(axis=-1), top[..., top_k]
    with np.errstate(divide="ignore", invalid="ignore"):
        return np.where(m_k > 0, (m_k - m_next) / m_k, 0.0)


def bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
