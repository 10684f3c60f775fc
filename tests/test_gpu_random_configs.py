"""Randomised differential test: seeded draws of shape, group size, salient mode, tiers, recent window, fused rotary
embedding, rotation flags and the way the rows are appended (pieces, then single-row decode steps); after every append
the cache is compared bit for bit with the oracle's, and decode attention within the tolerance, through the C ABI."""
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


def _compare(oc, gc, what):
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
    if oc.fine_mask is not None:
        assert np.array_equal(_u32(gc.fine_mask), oc.fine_mask), f"{what}: fine mask"


def _one_case(orc, case):
    rng = np.random.default_rng(7000 + case)
    Hkv = int(rng.integers(1, 4))
    R = int(rng.choice([1, 1, 2, 4, 7, 8]))
    Hq = Hkv * R
    B = int(rng.integers(1, 4))
    G = int(rng.choice([64, 128]))
    T = int(rng.integers(3, 260)) if case % 5 else int(rng.integers(260, 700))
    n_head = int(rng.integers(1, max(2, min(20, T - 2))))
    n_tail = int(rng.integers(1, max(2, min(12, T - n_head))))
    W_score = 16
    w = synth.small(f"rnd{case}", B=B, Hq=Hq, Hkv=Hkv, T=T, G=G, n_text_head=n_head, n_text_tail=n_tail,
                    top_k=int(rng.integers(1, 9)), W=W_score)
    d = {k: (v.numpy() if hasattr(v, "numpy") else v) for k, v in synth.generate(w, seed=900 + case).items()}
    window = int(rng.choice([0, 0, 64, 128]))
    tiered = bool(rng.integers(0, 2))
    rope = bool(rng.integers(0, 2))
    rot_v = bool(rng.integers(0, 4))          # mostly the method; sometimes V arrives rotated
    mode = str(rng.choice(["tsa", "psa", "none"])) if not tiered else "pivots"
    what = f"case {case}: B={B} Hq={Hq} Hkv={Hkv} G={G} T={T} window={window} tiered={tiered} rope={rope} " \
           f"rot_v={rot_v} mode={mode}"
    print(what, flush=True)
    flags_w = 0 if rot_v else akvq.V_PREROTATED
    flags_r = 0 if rot_v else akvq.OUT_ROTATED

    n_steps = int(rng.integers(0, 4)) if T > 8 else 0        # rows appended one at a time at the end
    T0 = T - n_steps
    if tiered:
        keep = [sorted(set(int(x) for x in d["pivots"][b] if x < T0)) for b in range(B)]
        row_src, row_tier, row_of = synth.tiered_rows(d["is_text"][:, :T0], keep)
        n_rows = row_src.shape[1]
    else:
        n_rows = T0
    t_cap = (n_rows + n_steps + 63) // 64 * 64
    oc = orc.OracleCache(B, Hkv, G, t_cap, 64, fill=0)
    gc = akvq.Cache(B, Hkv, G, t_cap, 64, fill=0)
    if window:
        oc.enable_window(window)
        gc.enable_window(window)
    if mode == "tsa":
        oc.select_tsa(d["is_text"][:, :T0])
    elif mode == "psa" and T0 >= W_score:
        oc.select_psa(d["q_tail"], d["k"][:, :, :T0], w.top_k, w.sm_scale)
    elif mode == "pivots":
        for b in range(B):
            rows = sorted(int(row_of[b, t]) for t in keep[b])
            oc.sal_idx[b, :, :len(rows)] = rows
            oc.sal_cnt[b, :] = len(rows)
    if n_steps and rng.integers(0, 2):       # list the last appended row as salient ahead of time
        for b in range(B):
            for h in range(Hkv):
                n = int(oc.sal_cnt[b, h])
                if n < 64:
                    oc.sal_idx[b, h, n] = n_rows + n_steps - 1
                    oc.sal_cnt[b, h] = n + 1
    gc.sal_idx.copy_(_dev(oc.sal_idx))
    gc.counts().copy_(_dev(oc.sal_cnt))

    pos = np.arange(T) + int(rng.integers(0, 50))
    cos_all, sin_all = synth.rope_tables(pos)

    def append(k, v, rs, rt, cos, sin):
        k_or = orc.rope_rows(k, cos, sin) if rope else k
        oc.quantize_append_tiered(k_or, v, rs, rt, w.clip, 1.0, rotate_v=rot_v)
        akvq.quantize_append_tiered(gc, _dev(k), _dev(v), None if rs is None else _dev(rs),
                                    None if rt is None else _dev(rt), w.clip, 1.0, flags=flags_w,
                                    rope=(_dev(cos), _dev(sin)) if rope else None)

    k0, v0 = d["k"][:, :, :T0], d["v"][:, :, :T0]
    if tiered:
        cuts = sorted(set([0, n_rows] + [2 * int(x) for x in rng.integers(0, n_rows // 2 + 1, size=2)]))
        for a, b_ in zip(cuts[:-1], cuts[1:]):
            append(k0, v0, np.ascontiguousarray(row_src[:, a:b_]), np.ascontiguousarray(row_tier[:, a:b_]),
                   cos_all[:T0], sin_all[:T0])
            _compare(oc, gc, f"{what}, rows {a}..{b_}")
    else:
        cuts = sorted(set([0, T0] + [int(x) for x in rng.integers(0, T0 + 1, size=2)]))
        for a, b_ in zip(cuts[:-1], cuts[1:]):
            append(k0[:, :, a:b_], v0[:, :, a:b_], None, None, cos_all[a:b_], sin_all[a:b_])
            _compare(oc, gc, f"{what}, rows {a}..{b_}")
    for t in range(T0, T):
        append(d["k"][:, :, t:t + 1], d["v"][:, :, t:t + 1], None, None, cos_all[t:t + 1], sin_all[t:t + 1])
        _compare(oc, gc, f"{what}, step {t}")

    cq, sq = synth.rope_tables(pos[-1:] + 1)
    q_or = orc.rope_rows(d["q"][:, :, None, :], cq, sq)[:, :, 0, :] if rope else d["q"]
    ref, lse_ref = oc.decode(q_or, w.sm_scale, unrotate=rot_v)
    for ns in (0, int(rng.integers(1, 6))):
        out, lse = akvq.decode_attention(gc, _dev(d["q"]), w.sm_scale, n_split=ns, flags=flags_r,
                                         rope=(_dev(cq), _dev(sq)) if rope else None)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        rel = np.abs(got - ref).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-6)
        assert rel.max() <= ATTN_TOL, f"{what}, n_split={ns}: {rel.max():.3e}"
        assert np.abs(lse.cpu().numpy() - lse_ref).max() <= 2e-3, what


@pytest.mark.parametrize("block", range(12))
def test_random_configurations(orc, block):
    for case in range(block * 8, block * 8 + 8):
        _one_case(orc, case)


@pytest.mark.parametrize("block", range(4))
def test_random_pivot_selection(orc, block):
    """Seeded draws for the attention-mass pivot selection: scoring rows 16..64, 1 to 8 query heads per kv-head,
    context lengths around the 2048-key chunk and 16-key group boundaries, top-k from 1 to 64."""
    from test_gpu_parity import check_psa
    for case in range(block * 6, block * 6 + 6):
        rng = np.random.default_rng(8100 + case)
        Hkv = int(rng.integers(1, 3))
        R = int(rng.choice([1, 2, 3, 7, 8]))
        W = int(rng.choice([16, 32, 48, 64]))
        T = int(rng.choice([W, W + 1, 2047, 2048, 2049, 4096 + 17, int(rng.integers(W, 3000))]))
        top_k = int(min(T, rng.choice([1, 4, 16, 64])))
        n_head = max(1, min(8, T // 4))
        w = synth.small(f"psa_rnd{case}", B=int(rng.integers(1, 3)), Hq=Hkv * R, Hkv=Hkv, T=max(T, 3), W=W, top_k=top_k,
                        n_text_head=n_head, n_text_tail=1)
        print(f"case {case}: B={w.B} Hq={w.Hq} Hkv={Hkv} T={w.T} W={W} top_k={top_k}", flush=True)
        check_psa(orc, w, 950 + 100 * case, top_k)     # the seed search may move on by a few seeds: keep the cases apart
