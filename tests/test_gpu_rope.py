"""GPU parity of the rotary position embedding fused in front of the rotation (Section III-C.2, Fig. 6):
akvq_quantize_append_rope on pre-RoPE K rows and akvq_decode_attention_rope on pre-RoPE queries against the oracle's
embedding followed by its ordinary write / read path, through the C ABI."""
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


def _assert_cache_equal(oc, gc, what):
    torch.cuda.synchronize()
    T = oc.T_len
    nb = (T + 31) // 32
    for name in ("k_codes", "v_codes"):
        assert np.array_equal(_u32(getattr(gc, name))[:, :, :nb], getattr(oc, name)[:, :, :nb]), f"{what} {name}"
    for name in ("k_meta", "v_meta"):
        assert np.array_equal(_u32(getattr(gc, name))[:, :, :T], getattr(oc, name)[:, :, :T]), f"{what} {name}"
    for name in ("k_sal", "v_sal"):
        got = getattr(gc, name).cpu().numpy().view(np.uint16).reshape(-1)
        assert np.array_equal(got, getattr(oc, name).reshape(-1)), f"{what} {name}"


def _check_decode(orc, oc, gc, q, pos, w, what, n_splits=(1, 3), per_batch=False):
    """q is pre-RoPE; every batch element sits at its own position when per_batch."""
    cos, sin = synth.rope_tables(np.asarray(pos)[:, None] if per_batch else np.asarray(pos[:1]))
    q_emb = orc.rope_rows(q[:, :, None, :], cos, sin)[:, :, 0, :]
    ref, lse_ref = oc.decode(q_emb, w.sm_scale)
    for ns in n_splits:
        out, lse = akvq.decode_attention(gc, _dev(q), w.sm_scale, n_split=ns, rope=(_dev(cos), _dev(sin)))
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        rel = np.abs(got - ref).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-6)
        assert rel.max() <= ATTN_TOL, f"{what} n_split={ns}: {rel.max():.3e}"
        assert np.abs(lse.cpu().numpy() - lse_ref).max() <= 2e-3, what


@pytest.mark.parametrize("Hq,Hkv,G,per_batch", [(3, 3, 128, False), (2, 2, 64, True), (8, 2, 128, True), (14, 2, 64, False)])
def test_rope_prefill_then_decode_steps(orc, Hq, Hkv, G, per_batch):
    """Prefill of pre-RoPE K (several blocks and a ragged tail), three single-row decode appends, decode attention with
    a pre-RoPE query after each; text tokens salient."""
    w = synth.small(f"rope{Hq}_{G}", B=2, Hq=Hq, Hkv=Hkv, T=150, G=G, n_text_head=9, n_text_tail=6, top_k=5, W=16)
    d = _np(synth.generate(w, seed=171))
    T0 = 147
    start = np.array([0, 37]) if per_batch else np.array([5, 5])          # first position of each batch element
    pos = start[:, None] + np.arange(w.T)[None, :]
    oc = orc.OracleCache(w.B, w.Hkv, G, 192, 64, fill=0)
    gc = akvq.Cache(w.B, w.Hkv, G, 192, 64, fill=0)
    oc.select_tsa(d["is_text"])
    gc.sal_idx.copy_(_dev(oc.sal_idx))
    gc.counts().copy_(_dev(oc.sal_cnt))

    def append(lo, hi):
        cos, sin = synth.rope_tables(pos[:, lo:hi] if per_batch else pos[0, lo:hi])
        k, v = d["k"][:, :, lo:hi], d["v"][:, :, lo:hi]
        oc.quantize_append(orc.rope_rows(k, cos, sin), v, w.clip)
        akvq.quantize_append_tiered(gc, _dev(k), _dev(v), None, None, w.clip, 1.0, rope=(_dev(cos), _dev(sin)))
        _assert_cache_equal(oc, gc, f"rows {lo}..{hi}")

    append(0, T0)
    rng = np.random.default_rng(3)
    for t in range(T0, w.T):
        append(t, t + 1)
        q = rng.standard_normal((w.B, Hq, 128)).astype(np.float16)
        _check_decode(orc, oc, gc, q, pos[:, t], w, f"after row {t}", per_batch=per_batch)


def test_rope_with_tiers_and_window(orc):
    """Pre-RoPE K through the tiered append with the recent window: the table row of a cache row is its source token's."""
    w = synth.small("rope_tw", B=2, Hq=4, Hkv=2, T=140, G=128, n_text_head=11, n_text_tail=7, top_k=4, W=16)
    d = _np(synth.generate(w, seed=172))
    keep = [sorted(set(int(x) for x in d["pivots"][b])) for b in range(w.B)]
    row_src, row_tier, row_of = synth.tiered_rows(d["is_text"], keep)
    n_rows = row_src.shape[1]
    t_cap = (n_rows + 63) // 64 * 64
    oc = orc.OracleCache(w.B, w.Hkv, 128, t_cap, 64, fill=0)
    gc = akvq.Cache(w.B, w.Hkv, 128, t_cap, 64, fill=0)
    oc.enable_window(64)
    gc.enable_window(64)
    for b in range(w.B):
        rows = sorted(int(row_of[b, t]) for t in keep[b])
        oc.sal_idx[b, :, :len(rows)] = rows
        oc.sal_cnt[b, :] = len(rows)
    gc.sal_idx.copy_(_dev(oc.sal_idx))
    gc.counts().copy_(_dev(oc.sal_cnt))
    cos, sin = synth.rope_tables(np.arange(w.T))
    oc.quantize_append_tiered(orc.rope_rows(d["k"], cos, sin), d["v"], row_src, row_tier, w.clip, 1.0)
    akvq.quantize_append_tiered(gc, _dev(d["k"]), _dev(d["v"]), _dev(row_src), _dev(row_tier), w.clip, 1.0,
                                rope=(_dev(cos), _dev(sin)))
    _assert_cache_equal(oc, gc, "tiered + window + rope")
    assert np.array_equal(_u32(gc.fine_mask), oc.fine_mask)
    for name in ("k_win", "v_win"):
        got = getattr(gc, name).cpu().numpy().view(np.uint16).reshape(-1)
        assert np.array_equal(got, getattr(oc, name).reshape(-1)), name
    _check_decode(orc, oc, gc, d["q"], np.array([w.T, w.T]), w, "tiered + window + rope", n_splits=(0, 2))


@pytest.mark.parametrize("G", [128, 64])
def test_rope_long_salient_list_with_window(orc, G):
    """Pre-RoPE K, a salient list of several overlay tiles (every other token plus a dense run) and a recent window, in
    pieces: the overlay rows come from the pass behind the block kernel, which applies the embedding itself, next to
    ring stores of the windowed instantiation."""
    T = 420
    w = synth.small(f"rope_list{G}", B=2, Hq=2, Hkv=2, T=T, G=G, n_text_head=9, n_text_tail=6, top_k=5, W=16)
    d = _np(synth.generate(w, seed=172))
    mask = np.zeros((w.B, T), dtype=np.uint8)
    mask[:, 1::2] = 1
    mask[:, 96:170] = 1
    n_sal = int(mask.sum(axis=1).max())
    s_cap = (n_sal + 63) // 64 * 64
    assert s_cap > 64
    oc = orc.OracleCache(w.B, w.Hkv, G, 448, s_cap, fill=0)
    gc = akvq.Cache(w.B, w.Hkv, G, 448, s_cap, fill=0)
    oc.enable_window(64); gc.enable_window(64)
    oc.select_tsa(mask)
    gc.sal_idx.copy_(_dev(oc.sal_idx))
    gc.counts().copy_(_dev(oc.sal_cnt))
    pos = np.array([3, 50])[:, None] + np.arange(T)[None, :]
    for lo, hi in ((0, 70), (70, 71), (71, 300), (300, 420)):
        cos, sin = synth.rope_tables(pos[:, lo:hi])
        k, v = d["k"][:, :, lo:hi], d["v"][:, :, lo:hi]
        oc.quantize_append_tiered(orc.rope_rows(k, cos, sin), v, None, None, w.clip, 1.0)
        akvq.quantize_append_tiered(gc, _dev(k), _dev(v), None, None, w.clip, 1.0, rope=(_dev(cos), _dev(sin)))
        _assert_cache_equal(oc, gc, f"rows {lo}..{hi}")
    rng = np.random.default_rng(4)
    q = rng.standard_normal((w.B, 2, 128)).astype(np.float16)
    _check_decode(orc, oc, gc, q, pos[:, T - 1] + 1, w, "long list + window + rope", per_batch=True)


def test_rope_rejects_prerotated_inputs():
    gc = akvq.Cache(1, 1, 128, 64, 64)
    k = torch.zeros(1, 1, 4, 128, dtype=torch.float16, device="cuda")
    cos = torch.ones(4, 64, dtype=torch.float16, device="cuda")
    with pytest.raises(akvq.AkvqError):
        akvq.quantize_append_tiered(gc, k, k, None, None, 0.8, 1.0, flags=akvq.K_PREROTATED, rope=(cos, cos))
    gc.T_len = 4
    q = torch.zeros(1, 1, 128, dtype=torch.float16, device="cuda")
    with pytest.raises(akvq.AkvqError):
        akvq.decode_attention(gc, q, 0.1, flags=akvq.Q_PREROTATED, rope=(cos[:1], cos[:1]))
