"""GPU parity of the 4-bit text tier (Section III-C.1) stored as row pairs: tiered append bit-exact against the
oracle, decode over the paired rows within the attention tolerance, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2501_15021_amd import binding as akvq
from paper_2501_15021_amd import synth

pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3


def _np(d):
    return {k: (v.cpu().numpy() if hasattr(v, "cpu") else v) for k, v in d.items()}


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _case(orc, w, seed, extra_text=True, pivots=True):
    d = _np(synth.generate(w, seed=seed))
    mask = d["is_text"].copy()
    if extra_text:
        mask[0, 40:47] = 1          # a run starting on an even position and one on an odd position
        mask[-1, 61:64] = 1
    keep = [sorted(set(int(x) for x in d["pivots"][b])) for b in range(w.B)] if pivots else None
    row_src, row_tier, row_of = synth.tiered_rows(mask, keep)
    n_rows = row_src.shape[1]
    t_cap = (n_rows + 63) // 64 * 64
    oc = orc.OracleCache(w.B, w.Hkv, w.G, t_cap, 64, fill=0)
    gc = akvq.Cache(w.B, w.Hkv, w.G, t_cap, 64, fill=0)
    if pivots:  # pivot tokens stay 16-bit: their rows are listed as salient (ascending rows)
        for b in range(w.B):
            rows = sorted(int(row_of[b, t]) for t in keep[b])
            oc.sal_idx[b, :, :len(rows)] = rows
            oc.sal_cnt[b, :] = len(rows)
        gc.sal_idx.copy_(_dev(oc.sal_idx))
        gc.counts().copy_(_dev(oc.sal_cnt))
    return d, row_src, row_tier, oc, gc


def _assert_equal(oc, gc, what):
    torch.cuda.synchronize()
    T = oc.T_len
    assert gc.T_len == T
    for name in ("k_codes", "v_codes"):
        got, ref = _u32(getattr(gc, name))[:, :, : (T + 31) // 32], getattr(oc, name)[:, :, : (T + 31) // 32]
        bad = np.argwhere(got != ref)
        assert bad.size == 0, f"{what} {name}: {len(bad)} words differ, first at {bad[0]}"
    for name in ("k_meta", "v_meta"):
        got, ref = _u32(getattr(gc, name))[:, :, :T], getattr(oc, name)[:, :, :T]
        bad = np.argwhere(got != ref)
        assert bad.size == 0, f"{what} {name}: {len(bad)} words differ, first at {bad[0]}: " \
                              f"{got[tuple(bad[0])]:#x} vs {ref[tuple(bad[0])]:#x}"
    for name in ("k_sal", "v_sal"):
        got = getattr(gc, name).cpu().numpy().view(np.uint16).reshape(-1)
        assert np.array_equal(got, getattr(oc, name).reshape(-1)), f"{what} {name}"
    assert np.array_equal(_u32(gc.fine_mask), oc.fine_mask), f"{what} fine mask"


@pytest.mark.parametrize("G", [128, 64])
def test_tiered_append_bit_exact(orc, G):
    w = synth.small(f"tier{G}", B=2, Hq=3, Hkv=3, T=150, G=G, n_text_head=9, n_text_tail=6)
    d, row_src, row_tier, oc, gc = _case(orc, w, seed=301 + G)
    oc.quantize_append_tiered(d["k"], d["v"], row_src, row_tier, 0.8, 1.0)
    akvq.quantize_append_tiered(gc, _dev(d["k"]), _dev(d["v"]), _dev(row_src), _dev(row_tier), 0.8, 1.0)
    assert (row_tier == 2).sum() > 20 and (row_tier == 3).sum() > 0
    _assert_equal(oc, gc, f"G={G}")


def test_tiered_append_in_pieces(orc):
    w = synth.small("tierp", B=2, Hq=2, Hkv=2, T=120, G=128, n_text_head=7, n_text_tail=5)
    d, row_src, row_tier, oc, gc = _case(orc, w, seed=311)
    n_rows = row_src.shape[1]
    cuts = [0, 10, 42, 44, 90, n_rows]            # all even, so no pair is split
    for a, b in zip(cuts[:-1], cuts[1:]):
        rs, rt = np.ascontiguousarray(row_src[:, a:b]), np.ascontiguousarray(row_tier[:, a:b])
        oc.quantize_append_tiered(d["k"], d["v"], rs, rt, 0.8, 1.0)
        akvq.quantize_append_tiered(gc, _dev(d["k"]), _dev(d["v"]), _dev(rs), _dev(rt), 0.8, 1.0)
    _assert_equal(oc, gc, "pieces")


def _decode_case(orc, w, seed, n_splits):
    d, row_src, row_tier, oc, gc = _case(orc, w, seed=seed)
    oc.quantize_append_tiered(d["k"], d["v"], row_src, row_tier, 0.8, 1.0)
    akvq.quantize_append_tiered(gc, _dev(d["k"]), _dev(d["v"]), _dev(row_src), _dev(row_tier), 0.8, 1.0)
    _assert_equal(oc, gc, w.name)
    ref, lse_ref = oc.decode(d["q"], w.sm_scale)
    q = _dev(d["q"])
    for ns in n_splits:
        out, lse = akvq.decode_attention(gc, q, w.sm_scale, n_split=ns)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        rel = np.abs(got - ref).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-6)
        assert rel.max() <= ATTN_TOL, f"{w.name} n_split={ns}: {rel.max():.3e}"
        assert np.abs(lse.cpu().numpy() - lse_ref).max() <= 2e-3


@pytest.mark.parametrize("G", [128, 64])
def test_tiered_decode_mha(orc, G):
    w = synth.small(f"tdm{G}", B=2, Hq=3, Hkv=3, T=210, G=G, n_text_head=21, n_text_tail=10, W=16)
    _decode_case(orc, w, 321 + G, (1, 3))


@pytest.mark.parametrize("Hq,Hkv,G", [(4, 2, 128), (14, 2, 64)])
def test_tiered_decode_gqa(orc, Hq, Hkv, G):
    w = synth.small(f"tdg{Hq}", B=2, Hq=Hq, Hkv=Hkv, T=333, G=G, n_text_head=33, n_text_tail=12, W=16)
    _decode_case(orc, w, 331 + Hq, (1, 4))


def test_tiered_cfg1(orc):
    w = synth.WORKLOADS["cfg1"]
    _decode_case(orc, w, 341, (0,))


# ---------------------------------------------------------------------------------------- recent window
def _assert_rings_equal(oc, gc, what):
    torch.cuda.synchronize()
    for name in ("k_win", "v_win"):
        got = getattr(gc, name).cpu().numpy().view(np.uint16).reshape(-1)
        assert np.array_equal(got, getattr(oc, name).reshape(-1)), f"{what} {name}"


def _check_decode(oc, gc, d, w, what, n_splits=(0,)):
    ref, lse_ref = oc.decode(d["q"], w.sm_scale)
    q = _dev(d["q"])
    for ns in n_splits:
        out, lse = akvq.decode_attention(gc, q, w.sm_scale, n_split=ns)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        rel = np.abs(got - ref).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-6)
        assert rel.max() <= ATTN_TOL, f"{what} n_split={ns}: {rel.max():.3e}"
        assert np.abs(lse.cpu().numpy() - lse_ref).max() <= 2e-3, what


@pytest.mark.parametrize("Hq,Hkv,G,W", [(3, 3, 128, 64), (3, 3, 64, 128), (8, 2, 128, 64), (14, 2, 64, 128)])
def test_window_prefill_then_decode_steps(orc, Hq, Hkv, G, W):
    """Prefill with a 16-bit recent window, then append rows one at a time: each step's attention must match the
    oracle, the rings must match bit for bit, and rows that left the window must be read from their codes."""
    w = synth.small(f"win{Hq}{G}", B=2, Hq=Hq, Hkv=Hkv, T=300, G=G, n_text_head=12, n_text_tail=8, top_k=6, W=16)
    d = _np(synth.generate(w, seed=401 + Hq + G))
    T0 = 230
    oc = orc.OracleCache(w.B, w.Hkv, w.G, 320, 64, fill=0)
    gc = akvq.Cache(w.B, w.Hkv, w.G, 320, 64, fill=0)
    oc.enable_window(W); gc.enable_window(W)
    oc.select_psa(d["q_tail"], d["k"][:, :, :T0], w.top_k, w.sm_scale)   # pivots of the prompt stay 16-bit as well
    gc.sal_idx.copy_(_dev(oc.sal_idx)); gc.counts().copy_(_dev(oc.sal_cnt))
    k0, v0 = d["k"][:, :, :T0], d["v"][:, :, :T0]
    oc.quantize_append_tiered(k0, v0, None, None, 0.8, 1.0)
    akvq.quantize_append_tiered(gc, _dev(k0), _dev(v0), None, None, 0.8, 1.0)
    _assert_equal_plain(oc, gc, "prefill")
    _assert_rings_equal(oc, gc, "prefill")
    _check_decode(oc, gc, d, w, "after prefill", (1, 3))
    for t in range(T0, w.T):
        kt, vt = d["k"][:, :, t:t + 1], d["v"][:, :, t:t + 1]
        oc.quantize_append_tiered(kt, vt, None, None, 0.8, 1.0)
        akvq.quantize_append_tiered(gc, _dev(kt), _dev(vt), None, None, 0.8, 1.0)
        if t in (T0, T0 + 1, T0 + 37, w.T - 1):
            _assert_rings_equal(oc, gc, f"step {t}")
            _check_decode(oc, gc, d, w, f"step {t}")
    _assert_equal_plain(oc, gc, "after the steps")


def _assert_equal_plain(oc, gc, what):
    torch.cuda.synchronize()
    T = oc.T_len
    assert gc.T_len == T
    for name in ("k_codes", "v_codes"):
        assert np.array_equal(_u32(getattr(gc, name)), getattr(oc, name)), f"{what} {name}"
    for name in ("k_meta", "v_meta"):
        assert np.array_equal(_u32(getattr(gc, name))[:, :, :T], getattr(oc, name)[:, :, :T]), f"{what} {name}"
    for name in ("k_sal", "v_sal"):
        got = getattr(gc, name).cpu().numpy().view(np.uint16).reshape(-1)
        assert np.array_equal(got, getattr(oc, name).reshape(-1)), f"{what} {name}"


def test_window_shorter_context_than_window(orc):
    w = synth.small("winshort", B=1, Hq=2, Hkv=2, T=50, G=128, W=16)
    d = _np(synth.generate(w, seed=431))
    oc = orc.OracleCache(w.B, w.Hkv, w.G, 64, 64, fill=0); gc = akvq.Cache(w.B, w.Hkv, w.G, 64, 64, fill=0)
    oc.enable_window(64); gc.enable_window(64)
    oc.quantize_append_tiered(d["k"], d["v"], None, None, 0.8, 1.0)
    akvq.quantize_append_tiered(gc, _dev(d["k"]), _dev(d["v"]), None, None, 0.8, 1.0)
    _assert_rings_equal(oc, gc, "short")
    _check_decode(oc, gc, d, w, "context shorter than the window")


@pytest.mark.parametrize("Hq,Hkv", [(3, 3), (8, 2)])
def test_window_with_four_bit_tier(orc, Hq, Hkv):
    """Tiers and window together: pairs inside the window are read once from the ring, pairs outside from their two
    rows; then a few decode steps with a text token (a pair) and a plain token appended."""
    w = synth.small(f"wint{Hq}", B=2, Hq=Hq, Hkv=Hkv, T=260, G=128, n_text_head=15, n_text_tail=30, W=16)
    d, row_src, row_tier, oc, gc = _case(orc, w, seed=441 + Hq)
    oc.enable_window(64); gc.enable_window(64)
    n_rows = row_src.shape[1]
    n0 = n_rows - 8
    a, b = np.ascontiguousarray(row_src[:, :n0]), np.ascontiguousarray(row_tier[:, :n0])
    oc.quantize_append_tiered(d["k"], d["v"], a, b, 0.8, 1.0)
    akvq.quantize_append_tiered(gc, _dev(d["k"]), _dev(d["v"]), _dev(a), _dev(b), 0.8, 1.0)
    _assert_equal(oc, gc, "tiered prefill")
    _assert_rings_equal(oc, gc, "tiered prefill")
    _check_decode(oc, gc, d, w, "tiered prefill", (1, 2))
    for lo in range(n0, n_rows, 2):      # two rows at a time: a pair, or two plain / padding rows
        a, b = np.ascontiguousarray(row_src[:, lo:lo + 2]), np.ascontiguousarray(row_tier[:, lo:lo + 2])
        oc.quantize_append_tiered(d["k"], d["v"], a, b, 0.8, 1.0)
        akvq.quantize_append_tiered(gc, _dev(d["k"]), _dev(d["v"]), _dev(a), _dev(b), 0.8, 1.0)
        _assert_rings_equal(oc, gc, f"rows {lo}")
        _check_decode(oc, gc, d, w, f"rows {lo}")
    _assert_equal(oc, gc, "tiered steps")
