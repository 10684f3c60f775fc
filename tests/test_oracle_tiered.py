"""Pins of the oracle's 4-bit text tier (Section III-C.1: text tokens 4-bit) and of its storage as row pairs.

None of these re-use the oracle's own formulas: the quantizer is checked against its error bound and a brute-force
nearest-level search, the pair format against the identity it must satisfy, and attention against a numpy
brute force over values dequantized directly from the 4-bit fields.
"""
import numpy as np
import pytest

from paper_2501_15021_amd import synth

D = 128


def _rows(seed, n, scale=1.0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, D)) * scale
    x[:, 5] *= 20.0
    return x.astype(np.float16)


@pytest.mark.parametrize("G", [128, 64])
def test_four_bit_quantizer_error_bound_and_nearest_level(orc, G):
    for i, row in enumerate(_rows(3, 40)):
        codes, sb, z, ybf = orc.quantize_row_bits(row, G, 1.0, 4)
        assert codes.max() <= 15
        y = orc.bf16_bits_to_f64(ybf)                    # rotated row (bf16-rounded: only used loosely below)
        u = orc.wht_dense(row.astype(np.float64))        # exact rotated row
        for g in range(D // G):
            s = float(sb[g:g + 1].view(np.float16)[0])
            sl = slice(g * G, (g + 1) * G)
            deq = s * (codes[sl].astype(np.float64) - float(z[g]))
            # clip 1: every value lies inside [min, max], so the error is at most half a step (plus fp32 slack)
            assert np.abs(deq - u[sl]).max() <= 0.5 * s * (1 + 2e-3) + 1e-6, (i, g)
            # the chosen level is the nearest of the 16 (ties aside)
            levels = s * (np.arange(16)[None, :] - float(z[g]))
            best = np.abs(levels - u[sl][:, None]).min(axis=1)
            assert np.all(np.abs(deq - u[sl]) <= best + 1e-5 * s)
            # 15 steps span the range: the scale is range/15 rounded up to binary16
            rng_ = u[sl].max() - u[sl].min()
            assert rng_ / 15 * (1 - 1e-3) <= s <= rng_ / 15 * (1 + 2e-3)
        assert np.abs(y - u).max() <= np.abs(u).max() * 2 ** -8


def test_four_bit_is_finer_than_two_bit(orc):
    row = _rows(9, 1)[0]
    u = orc.wht_dense(row.astype(np.float64))
    err = {}
    for bits in (2, 4):
        codes, sb, z, _ = orc.quantize_row_bits(row, 128, 1.0, bits)
        s = float(sb.view(np.float16)[0])
        err[bits] = np.abs(s * (codes.astype(np.float64) - float(z[0])) - u).max()
    assert err[4] < err[2] / 4


def _tiered_case(orc, G, rotate_v=True):
    """6 tokens -> 10 rows: [2-bit, pad, (coarse, fine), 2-bit, 2-bit, (coarse, fine), (coarse, fine)]"""
    B, H, n_src = 2, 2, 6
    rng = np.random.default_rng(17)
    k = (rng.standard_normal((B, H, n_src, D)) * 1.5).astype(np.float16)
    v = rng.standard_normal((B, H, n_src, D)).astype(np.float16)
    row_src = np.array([[0, 0, 1, 1, 2, 3, 4, 4, 5, 5]] * B, dtype=np.int32)
    row_tier = np.array([[0, 3, 1, 2, 0, 0, 1, 2, 1, 2]] * B, dtype=np.uint8)
    oc = orc.OracleCache(B, H, G, 64, 64)
    oc.quantize_append_tiered(k, v, row_src, row_tier, 0.8, 1.0, rotate_v=rotate_v)
    return oc, k, v, row_src, row_tier


@pytest.mark.parametrize("G", [128, 64])
def test_pair_rows_reproduce_the_four_bit_value(orc, G):
    oc, k, v, row_src, row_tier = _tiered_case(orc, G)
    assert oc.T_len == 10
    assert oc.fine_mask[0, 0] == (1 << 3) | (1 << 7) | (1 << 9)
    ng = D // G
    for b in range(2):
        for h in range(2):
            for tensor, src in ((0, k), (1, v)):
                meta = oc.k_meta if tensor == 0 else oc.v_meta
                for t in (2, 6, 8):                                    # coarse rows
                    tok = row_src[b, t]
                    c4, sb, z4, _ = orc.quantize_row_bits(src[b, h, tok], G, 1.0, 4)
                    for e in range(0, D, 7):
                        g = e // G
                        hi, lo = oc.get_code(tensor, b, h, t, e), oc.get_code(tensor, b, h, t + 1, e)
                        mc, mf = int(meta[b, h, t, g]), int(meta[b, h, t + 1, g])
                        sc = float(np.array([mc & 0x7FFF], dtype=np.uint16).view(np.float16)[0])
                        sf = float(np.array([mf & 0x7FFF], dtype=np.uint16).view(np.float16)[0])
                        zc = np.int16(np.uint16(mc >> 16)); zf = np.int16(np.uint16(mf >> 16))
                        s4 = float(sb[g:g + 1].view(np.float16)[0])
                        assert sf == s4 and sc == 4 * s4 and 0 <= zf <= 3 and not (mc & 0x8000) and not (mf & 0x8000)
                        assert 4 * hi + lo == c4[e] and 4 * int(zc) + int(zf) == int(z4[g])
                        assert sc * (hi - int(zc)) + sf * (lo - int(zf)) == s4 * (int(c4[e]) - int(z4[g]))
                # the padding row is flagged and the plain rows match the plain quantizer
                assert int(meta[b, h, 1, 0]) & 0x8000
                c2, sb2, z2, _ = orc.quantize_row_bits(src[b, h, 0], G, 0.8, 2)
                assert all(oc.get_code(tensor, b, h, 0, e) == c2[e] for e in range(D))
                assert int(meta[b, h, 0, 0]) == int(sb2[0]) | (int(np.uint16(z2[0])) << 16)


@pytest.mark.parametrize("G", [128, 64])
def test_tiered_decode_equals_brute_force_over_direct_dequant(orc, G):
    oc, k, v, row_src, row_tier = _tiered_case(orc, G)
    B, H = 2, 2
    rng = np.random.default_rng(23)
    q = rng.standard_normal((B, H, D)).astype(np.float16)
    sm = 0.11
    out, lse = oc.decode(q, sm)
    tokens = [(0, 2), (1, 4), (2, 2), (3, 2), (4, 4), (5, 4)]        # (source token, bits); the padding row is no token
    for b in range(B):
        for h in range(H):
            kd, vd = [], []
            for tok, bits in tokens:
                for src, dst in ((k, kd), (v, vd)):
                    c, sb, z, _ = orc.quantize_row_bits(src[b, h, tok], G, 0.8 if bits == 2 else 1.0, bits)
                    s = sb.view(np.float16).astype(np.float64)
                    dst.append(np.repeat(s, G) * (c.astype(np.float64) - np.repeat(z.astype(np.float64), G)))
            kd, vd = np.array(kd), np.array(vd)
            qr = orc.wht_dense(q[b, h].astype(np.float64))
            sc = sm * kd @ qr
            p = np.exp(sc - sc.max()); p /= p.sum()
            ref = orc.wht_dense(p @ vd)
            assert np.abs(out[b, h] - ref).max() <= 1e-9 * max(1.0, np.abs(ref).max())
            assert abs(lse[b, h] - (sc.max() + np.log(np.exp(sc - sc.max()).sum()))) <= 1e-9


def test_zero_point_split_handles_negative_and_large_zero_points(orc):
    # a group far from the origin: z4 is large (positive or negative); floor/mod split must still recombine
    for off in (-900.0, 700.0):
        row = (np.linspace(0.0, 3.0, D) + off).astype(np.float16)
        k = row[None, None, None, :].repeat(1, axis=0)
        oc = orc.OracleCache(1, 1, 128, 64, 64)
        oc.quantize_append_tiered(k, k, np.array([[0, 0]], dtype=np.int32), np.array([[1, 2]], dtype=np.uint8),
                                  0.8, 1.0, rotate_v=False)
        c4, sb, z4, _ = orc.quantize_row_bits(row, 128, 1.0, 4, rotate=False)
        mc, mf = int(oc.v_meta[0, 0, 0, 0]), int(oc.v_meta[0, 0, 1, 0])
        zc, zf = int(np.int16(np.uint16(mc >> 16))), int(np.int16(np.uint16(mf >> 16)))
        assert 0 <= zf <= 3 and 4 * zc + zf == int(z4[0])


# ---------------------------------------------------------------------------------------- recent window
def _brute_window(orc, k, v, q, b, h, G, T, t_win, sm):
    kd, vd = [], []
    for t in range(T):
        for src, dst in ((k, kd), (v, vd)):
            c, sb, z, ybf = orc.quantize_row_bits(src[b, h, t], G, 0.8, 2)
            if t >= t_win:
                dst.append(orc.bf16_bits_to_f64(ybf))
            else:
                s = sb.view(np.float16).astype(np.float64)
                dst.append(np.repeat(s, G) * (c.astype(np.float64) - np.repeat(z.astype(np.float64), G)))
    kd, vd = np.array(kd), np.array(vd)
    sc = sm * kd @ orc.wht_dense(q[b, h].astype(np.float64))
    p = np.exp(sc - sc.max()); p /= p.sum()
    return orc.wht_dense(p @ vd)


@pytest.mark.parametrize("T,W", [(200, 64), (70, 64), (40, 64), (129, 128)])
def test_window_rows_are_read_sixteen_bit(orc, T, W):
    B, H, G = 1, 2, 128
    rng = np.random.default_rng(41 + T)
    k = (rng.standard_normal((B, H, T, D)) * 1.5).astype(np.float16)
    v = rng.standard_normal((B, H, T, D)).astype(np.float16)
    q = rng.standard_normal((B, H, D)).astype(np.float16)
    oc = orc.OracleCache(B, H, G, 256, 64)
    oc.enable_window(W)
    oc.quantize_append_tiered(k, v, None, None, 0.8, 1.0)
    out, _ = oc.decode(q, 0.1)
    t_win = (max(T - W, 0) + 1) & ~1          # the boundary sits on an even row
    for h in range(H):
        ref = _brute_window(orc, k, v, q, 0, h, G, T, t_win, 0.1)
        assert np.abs(out[0, h] - ref).max() <= 1e-9 * max(1.0, np.abs(ref).max())


def test_rows_leaving_the_window_fall_back_to_their_codes(orc):
    """Appending row by row (each new row overwrites the ring slot of the row that leaves the window) must give the
    same cache and the same attention as appending everything at once."""
    B, H, G, T, W = 1, 2, 64, 150, 64
    rng = np.random.default_rng(47)
    k = (rng.standard_normal((B, H, T, D)) * 1.5).astype(np.float16)
    v = rng.standard_normal((B, H, T, D)).astype(np.float16)
    q = rng.standard_normal((B, H, D)).astype(np.float16)
    one = orc.OracleCache(B, H, G, 192, 64); one.enable_window(W)
    one.quantize_append_tiered(k, v, None, None, 0.8, 1.0)
    step = orc.OracleCache(B, H, G, 192, 64); step.enable_window(W)
    step.quantize_append_tiered(k[:, :, :90], v[:, :, :90], None, None, 0.8, 1.0)
    for t in range(90, T):
        step.quantize_append_tiered(k[:, :, t:t + 1], v[:, :, t:t + 1], None, None, 0.8, 1.0)
        if t in (100, 127, 149):
            ref = orc.OracleCache(B, H, G, 192, 64); ref.enable_window(W)
            ref.quantize_append_tiered(k[:, :, :t + 1], v[:, :, :t + 1], None, None, 0.8, 1.0)
            a, _ = step.decode(q, 0.1); r, _ = ref.decode(q, 0.1)
            assert np.abs(a - r).max() <= 1e-12
    assert np.array_equal(step.k_codes, one.k_codes) and np.array_equal(step.v_meta, one.v_meta)
    assert np.array_equal(step.k_win, one.k_win) and np.array_equal(step.v_win, one.v_win)


def test_window_with_four_bit_pairs(orc):
    """Pairs inside the window are read from the ring once (the fine half carries nothing there); pairs outside are
    the sum of their halves; the padding row is no token anywhere."""
    B, H, G, W = 1, 1, 128, 64
    rng = np.random.default_rng(53)
    n_tok = 60
    k = (rng.standard_normal((B, H, n_tok, D)) * 1.5).astype(np.float16)
    v = rng.standard_normal((B, H, n_tok, D)).astype(np.float16)
    q = rng.standard_normal((B, H, D)).astype(np.float16)
    mask = np.zeros((B, n_tok), dtype=np.uint8); mask[0, 3:9] = 1; mask[0, 41:52] = 1
    row_src, row_tier, row_of = synth.tiered_rows(mask)
    n_rows = row_src.shape[1]
    oc = orc.OracleCache(B, H, G, 128, 64); oc.enable_window(W)
    oc.quantize_append_tiered(k, v, row_src, row_tier, 0.8, 1.0)
    out, _ = oc.decode(q, 0.1)
    t_win = (max(n_rows - W, 0) + 1) & ~1
    kd, vd = [], []
    for r in range(n_rows):
        tier, tok = int(row_tier[0, r]), int(row_src[0, r])
        if tier in (2, 3):
            continue
        for src, dst in ((k, kd), (v, vd)):
            bits, clip = (4, 1.0) if tier == 1 else (2, 0.8)
            c, sb, z, ybf = orc.quantize_row_bits(src[0, 0, tok], G, clip, bits)
            if r >= t_win:
                dst.append(orc.bf16_bits_to_f64(ybf))
            else:
                s = float(sb.view(np.float16)[0])
                dst.append(s * (c.astype(np.float64) - float(z[0])))
    kd, vd = np.array(kd), np.array(vd)
    sc = 0.1 * kd @ orc.wht_dense(q[0, 0].astype(np.float64))
    p = np.exp(sc - sc.max()); p /= p.sum()
    ref = orc.wht_dense(p @ vd)
    assert np.abs(out[0, 0] - ref).max() <= 1e-9 * max(1.0, np.abs(ref).max())
