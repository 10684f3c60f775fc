"""GPU parity of akvq_decode_step (one generated token in one launch: append the row, then attend over the cache
including it): after every step the cache equals the oracle's bit for bit, attention is within the tolerance, and with
one KV split the output equals the two separate calls bit for bit."""
import numpy as np
import pytest
import torch

from paper_2501_15021_amd import binding as akvq
from paper_2501_15021_amd import synth

pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _compare_cache(oc, gc, what):
    torch.cuda.synchronize()
    T = oc.T_len
    assert gc.T_len == T, what
    nb = (T + 31) // 32
    for name in ("k_codes", "v_codes"):
        assert np.array_equal(_u32(getattr(gc, name))[:, :, :nb], getattr(oc, name)[:, :, :nb]), f"{what}: {name}"
    for name in ("k_meta", "v_meta"):
        assert np.array_equal(_u32(getattr(gc, name))[:, :, :T], getattr(oc, name)[:, :, :T]), f"{what}: {name}"
    for name in ("k_sal", "v_sal") + (("k_win", "v_win") if oc.W else ()):
        got = getattr(gc, name).cpu().numpy().view(np.uint16).reshape(-1)
        assert np.array_equal(got, getattr(oc, name).reshape(-1)), f"{what}: {name}"


SPLITS = (1, 3, 4, 5)


@pytest.mark.parametrize("Hq,Hkv,G,window,rope,T0", [
    (3, 3, 128, 0, False, 150), (3, 3, 64, 64, True, 61), (2, 2, 128, 0, True, 0), (8, 2, 128, 128, False, 200),
    (14, 2, 64, 0, True, 97), (7, 1, 64, 64, False, 130), (4, 4, 128, 64, True, 255),
    # 5 tiles in 4 splits (runs of 2: the last split is empty and the third one owns the new row's tile)
    (2, 2, 128, 0, False, 262), (4, 2, 64, 0, False, 133)])
def test_decode_steps(orc, Hq, Hkv, G, window, rope, T0):
    """Every split count steps a cache of its own, so the row a step appends is still unwritten (zero) when the launch
    starts: a workgroup that read the row's tile without being the one that wrote it would see zeros and fail the
    attention comparison.  The shapes cover fewer tiles than splits, trailing empty splits and uneven runs."""
    n_steps = 6
    w = synth.small(f"step{Hq}_{G}", B=2, Hq=Hq, Hkv=Hkv, T=max(T0 + n_steps, 12), G=G, n_text_head=3, n_text_tail=2,
                    top_k=4, W=16)
    d = {k: (v.numpy() if hasattr(v, "numpy") else v) for k, v in synth.generate(w, seed=191 + Hq + T0).items()}
    t_cap = (w.T + 63) // 64 * 64
    oc = orc.OracleCache(w.B, Hkv, G, t_cap, 64, fill=0)
    gcs = {ns: akvq.Cache(w.B, Hkv, G, t_cap, 64, fill=0) for ns in SPLITS}
    ref_gc = akvq.Cache(w.B, Hkv, G, t_cap, 64, fill=0)       # the two separate calls, for the exact comparison
    every = [oc, ref_gc, *gcs.values()]
    for c in every:
        if window:
            c.enable_window(window)
    listed = np.array(sorted({1, max(T0 - 1, 2), T0 + 1, T0 + 4}), dtype=np.int32)     # two of the new rows are salient
    oc.sal_idx[:, :, :len(listed)] = listed
    oc.sal_cnt[:] = len(listed)
    for c in every[1:]:
        c.sal_idx.copy_(_dev(oc.sal_idx))
        c.counts().copy_(_dev(oc.sal_cnt))
    pos = np.arange(w.T) + 11
    cos_all, sin_all = synth.rope_tables(pos)
    if T0 > 0:
        k0, v0 = d["k"][:, :, :T0], d["v"][:, :, :T0]
        r0 = (cos_all[:T0], sin_all[:T0])
        oc.quantize_append_tiered(orc.rope_rows(k0, *r0) if rope else k0, v0, None, None, w.clip, 1.0)
        for c in every[1:]:
            akvq.quantize_append_tiered(c, _dev(k0), _dev(v0), None, None, w.clip, 1.0,
                                        rope=(_dev(r0[0]), _dev(r0[1])) if rope else None)
    rng = np.random.default_rng(T0)
    for t in range(T0, T0 + n_steps):
        k1, v1 = d["k"][:, :, t:t + 1], d["v"][:, :, t:t + 1]
        q = rng.standard_normal((w.B, Hq, 128)).astype(np.float16)
        r1 = (cos_all[t:t + 1], sin_all[t:t + 1])
        rd = (_dev(r1[0]), _dev(r1[1])) if rope else None
        oc.quantize_append_tiered(orc.rope_rows(k1, *r1) if rope else k1, v1, None, None, w.clip, 1.0)
        q_or = orc.rope_rows(q[:, :, None, :], *r1)[:, :, 0, :] if rope else q
        ref, lse_ref = oc.decode(q_or, w.sm_scale)
        for ns, gc in gcs.items():
            assert gc.T_len == t
            out, lse = akvq.decode_step(gc, _dev(k1), _dev(v1), _dev(q), w.clip, w.sm_scale, n_split=ns, rope=rd)
            _compare_cache(oc, gc, f"step {t}, n_split={ns}")
            got = out.cpu().numpy().astype(np.float64)
            rel = np.abs(got - ref).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-6)
            assert rel.max() <= ATTN_TOL, f"step {t}, n_split={ns}: {rel.max():.3e}"
            assert np.abs(lse.cpu().numpy() - lse_ref).max() <= 2e-3
            if ns == 1:
                ref_gc.T_len = t
                akvq.quantize_append_tiered(ref_gc, _dev(k1), _dev(v1), None, None, w.clip, 1.0, rope=rd)
                out2, lse2 = akvq.decode_attention(ref_gc, _dev(q), w.sm_scale, n_split=1, rope=rd)
                torch.cuda.synchronize()
                assert torch.equal(out, out2) and torch.equal(lse, lse2), f"step {t}: fused vs separate calls"


@pytest.mark.parametrize("Hq,Hkv,G,T0", [(2, 2, 128, 18436), (7, 1, 64, 34820)])
def test_decode_step_default_splits_with_an_empty_last_split(orc, Hq, Hkv, G, T0):
    """Long rows in few (batch, kv-head) units: the default split count leaves the last split without tiles (289 tiles
    in 18 runs of 17; 1089 in 68 -> 64 runs of 18), so the split that appends is not the last one."""
    w = synth.small(f"steplong{Hq}", B=1, Hq=Hq, Hkv=Hkv, T=T0 + 3, G=G, n_text_head=3, n_text_tail=2, top_k=4, W=16)
    L = akvq.lib()
    rows = 64 if Hq == Hkv else 32
    import ctypes as C
    b, e = C.c_int(), C.c_int()
    ns = L.akvq_decode_default_splits(w.B, Hkv, T0 + 1)
    owner = L.akvq_decode_split_range((T0 + rows) // rows, ns, ns - 1, C.byref(b), C.byref(e))
    assert owner < ns - 1 and b.value == e.value, "the shape is meant to leave the last split empty"
    d = {k: (v.numpy() if hasattr(v, "numpy") else v) for k, v in synth.generate(w, seed=195).items()}
    t_cap = (w.T + 63) // 64 * 64
    oc = orc.OracleCache(w.B, Hkv, G, t_cap, 64, fill=0)
    gc = akvq.Cache(w.B, Hkv, G, t_cap, 64, fill=0)
    oc.quantize_append(d["k"][:, :, :T0], d["v"][:, :, :T0], w.clip)
    akvq.quantize_append(gc, _dev(d["k"][:, :, :T0]), _dev(d["v"][:, :, :T0]), w.clip)
    rng = np.random.default_rng(3)
    for t in range(T0, T0 + 3):
        k1, v1 = d["k"][:, :, t:t + 1] * 3, d["v"][:, :, t:t + 1] * 50   # a row whose absence would show in the output
        q = (rng.standard_normal((w.B, Hq, 128)) + np.sign(k1[:, :1, 0, :].astype(np.float64))).astype(np.float16)
        oc.quantize_append(k1, v1, w.clip)
        ref, lse_ref = oc.decode(q, w.sm_scale)
        out, lse = akvq.decode_step(gc, _dev(k1), _dev(v1), _dev(q), w.clip, w.sm_scale, n_split=0)
        _compare_cache(oc, gc, f"long step {t}")
        got = out.cpu().numpy().astype(np.float64)
        rel = np.abs(got - ref).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-6)
        assert rel.max() <= ATTN_TOL, f"long step {t}: {rel.max():.3e}"
        assert np.abs(lse.cpu().numpy() - lse_ref).max() <= 2e-3


def test_decode_step_after_tiered_prefill(orc):
    """4-bit text pairs in the cache (the paired decode kernels), then fused steps with plain rows."""
    w = synth.small("step_tier", B=2, Hq=4, Hkv=2, T=140, G=128, n_text_head=11, n_text_tail=7, top_k=4, W=16)
    d = {k: (v.numpy() if hasattr(v, "numpy") else v) for k, v in synth.generate(w, seed=193).items()}
    T0 = 134
    row_src, row_tier, row_of = synth.tiered_rows(d["is_text"][:, :T0], [[0]] * w.B)
    n_rows = row_src.shape[1]
    t_cap = (n_rows + 6 + 63) // 64 * 64
    oc = orc.OracleCache(w.B, w.Hkv, 128, t_cap, 64, fill=0)
    gc = akvq.Cache(w.B, w.Hkv, 128, t_cap, 64, fill=0)
    oc.enable_window(64)
    gc.enable_window(64)
    oc.quantize_append_tiered(d["k"][:, :, :T0], d["v"][:, :, :T0], row_src, row_tier, w.clip, 1.0)
    akvq.quantize_append_tiered(gc, _dev(d["k"][:, :, :T0]), _dev(d["v"][:, :, :T0]), _dev(row_src), _dev(row_tier),
                                w.clip, 1.0)
    rng = np.random.default_rng(5)
    for t in range(T0, T0 + 6):
        k1, v1 = d["k"][:, :, t:t + 1], d["v"][:, :, t:t + 1]
        q = rng.standard_normal((w.B, w.Hq, 128)).astype(np.float16)
        oc.quantize_append_tiered(k1, v1, None, None, w.clip, 1.0)
        ref, _ = oc.decode(q, w.sm_scale)
        out, _ = akvq.decode_step(gc, _dev(k1), _dev(v1), _dev(q), w.clip, w.sm_scale, n_split=2)
        _compare_cache(oc, gc, f"tiered step {t}")
        got = out.cpu().numpy().astype(np.float64)
        rel = np.abs(got - ref).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-6)
        assert rel.max() <= ATTN_TOL, f"tiered step {t}: {rel.max():.3e}"


def test_decode_step_with_offline_fold_flags(orc):
    """V arrives rotated and the output stays rotated (Section III-C.2 offline mode): the fused step passes the write-
    and the read-path flags together."""
    w = synth.small("step_flags", B=2, Hq=4, Hkv=2, T=80, G=128, n_text_head=3, n_text_tail=2, top_k=4, W=16)
    d = {k: (v.numpy() if hasattr(v, "numpy") else v) for k, v in synth.generate(w, seed=197).items()}
    T0 = 75
    oc = orc.OracleCache(w.B, w.Hkv, 128, 128, 64, fill=0)
    gc = akvq.Cache(w.B, w.Hkv, 128, 128, 64, fill=0)
    oc.quantize_append(d["k"][:, :, :T0], d["v"][:, :, :T0], w.clip, rotate_v=False)
    akvq.quantize_append(gc, _dev(d["k"][:, :, :T0]), _dev(d["v"][:, :, :T0]), w.clip, flags=akvq.V_PREROTATED)
    rng = np.random.default_rng(9)
    for t in range(T0, w.T):
        k1, v1 = d["k"][:, :, t:t + 1], d["v"][:, :, t:t + 1]
        q = rng.standard_normal((w.B, w.Hq, 128)).astype(np.float16)
        oc.quantize_append(k1, v1, w.clip, rotate_v=False)
        ref, _ = oc.decode(q, w.sm_scale, unrotate=False)
        out, _ = akvq.decode_step(gc, _dev(k1), _dev(v1), _dev(q), w.clip, w.sm_scale, n_split=2,
                                  flags=akvq.V_PREROTATED | akvq.OUT_ROTATED)
        _compare_cache(oc, gc, f"flags step {t}")
        got = out.cpu().numpy().astype(np.float64)
        rel = np.abs(got - ref).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-6)
        assert rel.max() <= ATTN_TOL, f"flags step {t}: {rel.max():.3e}"
