"""How far this build's reading of the quantizer is from Eq. 3, 5 and 6 evaluated literally.

The oracle (and the GPU) take Eq. 5 as a multiply by the binary32 constant nearest to 1/3, and Eq. 3 as ONE rounding of
u * rcpu + zero (u the un-normalised butterfly value, rcpu = fl(fl(1/s) * 2^-3.5), the zero-point added before the
rounding).  Literally, Eq. 5 is a division by 2^n - 1 = 3 and Eq. 3 is round(X / scale) + zero with X the rotated value
and a true division.  This test evaluates the literal forms in binary32 with numpy (correctly rounded divisions, round
half to even) next to the oracle on every row of configuration 1 (K and V, clip 0.8 and 1.0, groups of 128 and 64) and
asserts that they differ only where the reading says they can:
  * a stored scale differs only when the two binary32 results differ (by one ulp) and straddle a binary16 rounding
    boundary: then by exactly one binary16 step;
  * with scale and zero-point equal, a code differs only when x / scale + zero lies within a few binary32 ulps of a
    half-way point (the four roundings of the literal form against the one of the reading);
  * a zero-point differs only when clipped_min / scale lies that close to a half-way point.
The counts are printed (pytest -s) and recorded in the design notes.
"""
import ctypes as C

import numpy as np
import pytest

from paper_2501_15021_amd import synth

KAPPA = np.array([0x3DB504F3], dtype=np.uint32).view(np.float32)[0]      # 2^-3.5 as binary32
F32 = np.float32


def fwht128_numpy_f32(x):
    """Stride 1, 2, ..., 64 butterflies in binary32, every add rounded on its own (rows of 128 along the last axis)."""
    u = np.array(x, dtype=np.float32)
    n = u.shape[-1]
    h = 1
    while h < n:
        v = u.reshape(*u.shape[:-1], n // (2 * h), 2, h)
        a, b = v[..., 0, :].copy(), v[..., 1, :].copy()
        v[..., 0, :] = a + b
        v[..., 1, :] = a - b
        u = v.reshape(*u.shape[:-1], n)
        h *= 2
    return u


def half_round_up(s32):
    """binary16 value not below s32 (round to nearest even, then one step up if that fell below); numpy's cast is
    pinned against the oracle's conversion on all patterns elsewhere."""
    s16 = s32.astype(np.float16)
    low = s16.astype(np.float32) < s32
    bits = s16.view(np.uint16) + low.astype(np.uint16)
    return bits


def oracle_rows(orc, rows_f16, G, clip):
    """The oracle's codes [n,128], scale bits [n,128/G], zero-points [n,128/G] of fp16 rows [n,128]."""
    L = orc.lib()
    n = rows_f16.shape[0]
    ng = 128 // G
    rows = np.ascontiguousarray(rows_f16).view(np.uint16)
    codes = np.zeros((n, 128), dtype=np.uint8)
    sb = np.zeros((n, ng), dtype=np.uint16)
    z = np.zeros((n, ng), dtype=np.int16)
    ybf = np.zeros(128, dtype=np.uint16)
    f = L.orc_quantize_row
    p_rows, p_codes, p_sb, p_z, p_y = (a.ctypes.data for a in (rows, codes, sb, z, ybf))
    for i in range(n):
        f(C.c_void_p(p_rows + 256 * i), G, C.c_float(clip), 1, C.c_void_p(p_codes + 128 * i),
          C.c_void_p(p_sb + 2 * ng * i), C.c_void_p(p_z + 2 * ng * i), C.c_void_p(p_y))
    return codes, sb, z


@pytest.mark.parametrize("G", [128, 64])
@pytest.mark.parametrize("clip", [0.8, 1.0])
def test_reading_differs_from_the_literal_equations_only_on_ties(orc, G, clip):
    w = synth.WORKLOADS["cfg1"]
    d = synth.generate(w)
    rows = np.concatenate([d["k"].numpy().reshape(-1, 128), d["v"].numpy().reshape(-1, 128)])   # 2 x 20480 rows
    n, ng = rows.shape[0], 128 // G
    codes_o, sb_o, z_o = oracle_rows(orc, rows, G, clip)

    u = fwht128_numpy_f32(rows.astype(np.float32))
    for i in (0, 1, n // 2, n - 1):                       # the numpy butterfly is the oracle's, bit for bit
        assert np.array_equal(u[i].view(np.uint32), orc.fwht128_f32(rows[i].astype(np.float32)).view(np.uint32))
    y = u * KAPPA                                          # X of Eq. 3: the rotated value, rounded to binary32
    yg = y.reshape(n, ng, G)
    cmin = F32(clip) * yg.min(-1)
    cmax = F32(clip) * yg.max(-1)
    rng = cmax - cmin
    s32_div = rng / F32(3.0)                               # Eq. 5, literally
    s32_mul = rng * np.array([0x3EAAAAAB], dtype=np.uint32).view(np.float32)[0]
    assert (rng > 0).all()
    sb_lit = half_round_up(s32_div)
    # ---- scale: the reading's multiply is within one binary32 ulp of the division; stored scales differ only there
    ulp = np.spacing(s32_div)
    assert (np.abs(s32_mul.astype(np.float64) - s32_div.astype(np.float64)) <= ulp).all()
    assert np.array_equal(half_round_up(s32_mul), sb_o), "the numpy replica of the reading must give the oracle's scale"
    scale_diff = sb_lit != sb_o
    assert (s32_mul[scale_diff] != s32_div[scale_diff]).all()
    assert (np.abs(sb_lit.astype(np.int32) - sb_o.astype(np.int32))[scale_diff] == 1).all()
    # ---- zero-point (Eq. 6) and codes (Eq. 3) on the groups whose stored scale agrees
    s = sb_o.view(np.float16).astype(np.float32)           # the stored scale; all later arithmetic uses it
    zq_lit = cmin / s                                      # literally: clipped_min / scale
    z_lit = -np.rint(zq_lit).astype(np.int64)
    zero_diff = (z_lit != z_o) & ~scale_diff
    zq64 = cmin.astype(np.float64) / s.astype(np.float64)
    tie_dist = np.abs(np.abs(zq64 - np.floor(zq64)) - 0.5)
    assert (tie_dist[zero_diff] <= 2.0 ** -21 * np.maximum(np.abs(zq64[zero_diff]), 1.0)).all()
    same = ~scale_diff & ~zero_diff
    q_lit = np.rint(yg / s[..., None]).astype(np.int64) + z_o[..., None]          # round(X / scale) + zero
    code_lit = np.clip(q_lit, 0, 3).astype(np.uint8)
    code_o = codes_o.reshape(n, ng, G)
    code_diff = (code_lit != code_o) & same[..., None]
    q64 = yg.astype(np.float64) / s.astype(np.float64)[..., None]
    dist = np.abs(np.abs(q64 - np.floor(q64)) - 0.5)
    assert (dist[code_diff] <= 2.0 ** -21 * np.maximum(np.abs(q64[code_diff]), 1.0)).all(), \
        "a code differs from the literal Eq. 3 away from a half-way point"
    assert (np.abs(code_lit.astype(np.int32) - code_o.astype(np.int32))[code_diff] == 1).all()
    n_groups, n_elems = n * ng, int(same.sum()) * G
    print(f"\nG={G} clip={clip}: {n_groups} groups: stored scale differs in {int(scale_diff.sum())} "
          f"(binary32 results differ in {int((s32_mul != s32_div).sum())}), zero-point in {int(zero_diff.sum())}; "
          f"codes differ in {int(code_diff.sum())} of {n_elems} elements with equal scale and zero-point")
    # the differences are rare: well under one element in ten thousand, one group in a hundred
    assert code_diff.sum() <= 1e-4 * n_elems and scale_diff.sum() <= 1e-2 * n_groups and zero_diff.sum() <= 1e-3 * n_groups
