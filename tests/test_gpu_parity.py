"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.

Bars: packed codes, meta words (scale / zero / salient bit), overlay rows and salient index sets bit-exact;
attention output within 2e-3 of the oracle relative to the row's largest output magnitude (fp32 accumulation).
"""
import numpy as np
import pytest
import torch

import psa_inputs
from paper_2501_15021_amd import binding as akvq
from paper_2501_15021_amd import synth

pytestmark = pytest.mark.gpu

D = 128
ATTN_TOL = 2e-3


def _np(d):
    return {k: (v.cpu().numpy() if hasattr(v, "cpu") else v) for k, v in d.items()}


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _u16(t):
    return t.cpu().numpy().view(np.uint16)


def make_pair(orc, w, fill=0, t_cap=None, s_cap=None, layer=0):
    t_cap = t_cap or (w.T + 63) // 64 * 64
    s_cap = s_cap or w.s_cap(layer)
    oc = orc.OracleCache(w.B, w.Hkv, w.G, t_cap, s_cap, fill=fill)
    gc = akvq.Cache(w.B, w.Hkv, w.G, t_cap, s_cap, fill=fill)
    return oc, gc


def copy_salient_to_gpu(oc, gc):
    gc.sal_idx.copy_(_dev(oc.sal_idx))
    gc.counts().copy_(_dev(oc.sal_cnt))


def assert_cache_equal(oc, gc, what=""):
    T = oc.T_len
    assert gc.T_len == T
    torch.cuda.synchronize()
    for name in ("k_codes", "v_codes"):
        got, ref = _u32(getattr(gc, name)), getattr(oc, name)
        bad = np.argwhere(got != ref)
        assert bad.size == 0, f"{what} {name}: {len(bad)} words differ, first at {bad[0]}: " \
                              f"{got[tuple(bad[0])]:#x} vs {ref[tuple(bad[0])]:#x}"
    for name in ("k_meta", "v_meta"):
        got, ref = _u32(getattr(gc, name))[:, :, :T], getattr(oc, name)[:, :, :T]
        bad = np.argwhere(got != ref)
        assert bad.size == 0, f"{what} {name}: {len(bad)} words differ, first at {bad[0]}: " \
                              f"{got[tuple(bad[0])]:#x} vs {ref[tuple(bad[0])]:#x}"
    for name in ("k_sal", "v_sal"):
        got, ref = _u16(getattr(gc, name)), getattr(oc, name)
        bad = np.argwhere(got != ref)
        assert bad.size == 0, f"{what} {name}: {len(bad)} values differ, first at {bad[0]}"


def assert_attention_close(out_gpu, lse_gpu, out_ref, lse_ref, what="", lse_tol=2e-3):
    out_gpu = out_gpu.cpu().numpy().astype(np.float64)
    err = np.abs(out_gpu - out_ref).max(axis=-1)
    scale = np.maximum(np.abs(out_ref).max(axis=-1), 1e-6)
    rel = err / scale
    worst = np.unravel_index(np.argmax(rel), rel.shape)
    assert rel.max() <= ATTN_TOL, f"{what}: worst relative error {rel.max():.3e} at (b,h)={worst}"
    if lse_gpu is not None:
        assert np.abs(lse_gpu.cpu().numpy() - lse_ref).max() <= lse_tol, what
    return rel.max()


# ------------------------------------------------------------------------------------------- write path
@pytest.mark.parametrize("G,T,clip,fill", [(128, 70, 0.8, 0), (64, 70, 1.0, 0xFF), (128, 640, 0.8, 0),
                                           (64, 193, 0.8, 0xA5), (128, 1, 0.8, 0)])
def test_quantize_append_bit_exact(orc, G, T, clip, fill):
    w = synth.small(f"q{G}_{T}", B=2, Hq=3, Hkv=3, T=max(T, 12), G=G, clip=clip)
    d = _np(synth.generate(w, seed=101 + T))
    k, v = d["k"][:, :, :T], d["v"][:, :, :T]
    oc, gc = make_pair(orc, w, fill=fill, t_cap=(T + 63) // 64 * 64 + 64, s_cap=64)
    oc.select_tsa(d["is_text"])
    copy_salient_to_gpu(oc, gc)
    oc.quantize_append(k, v, clip)
    akvq.quantize_append(gc, _dev(k), _dev(v), clip)
    assert_cache_equal(oc, gc, f"G={G} T={T}")


@pytest.mark.parametrize("T,every", [(700, 3), (2304, 1), (1500, 7)])
def test_quantize_long_salient_lists(orc, T, every):
    """Salient lists longer than one wavefront: the kernel locates a block's run of entries by sampling the list
    (and by a plain scan beyond 2048 entries); slots and overlay rows must still match the oracle exactly."""
    w = synth.small(f"qlist{T}", B=1, Hq=2, Hkv=2, T=T, G=128)
    d = _np(synth.generate(w, seed=77 + T))
    mask = np.zeros((w.B, T), dtype=np.uint8)
    mask[:, ::every] = 1
    mask[:, 5:40] = 1  # a dense run inside the first blocks
    n_sal = int(mask[0].sum())
    oc, gc = make_pair(orc, w, t_cap=(T + 63) // 64 * 64, s_cap=(n_sal + 63) // 64 * 64)
    oc.select_tsa(mask)
    copy_salient_to_gpu(oc, gc)
    oc.quantize_append(d["k"], d["v"], 0.8)
    akvq.quantize_append(gc, _dev(d["k"]), _dev(d["v"]), 0.8)
    assert_cache_equal(oc, gc, f"T={T} every={every} salient={n_sal}")


def test_quantize_long_salient_list_in_pieces(orc):
    """A long salient list filled over several appends: overlay tiles then hold rows of earlier appends next to the new
    ones (and unused slots, pre-filled with a pattern), which the overlay pass must leave as they are."""
    T = 900
    w = synth.small("qlist_pieces", B=2, Hq=2, Hkv=2, T=T, G=64)
    d = _np(synth.generate(w, seed=81))
    mask = np.zeros((w.B, T), dtype=np.uint8)
    mask[:, ::2] = 1
    mask[:, 130:260] = 1
    mask[1, 600:] = 0  # the batch elements differ
    n_sal = int(mask.sum(axis=1).max())
    oc, gc = make_pair(orc, w, fill=0x5A, t_cap=(T + 63) // 64 * 64, s_cap=(n_sal + 63) // 64 * 64)
    oc.select_tsa(mask)
    copy_salient_to_gpu(oc, gc)
    cuts = [0, 33, 34, 100, 163, 164, 512, 899, 900]
    for a, b in zip(cuts[:-1], cuts[1:]):
        oc.quantize_append(d["k"][:, :, a:b], d["v"][:, :, a:b], 0.8)
        akvq.quantize_append(gc, _dev(d["k"][:, :, a:b]), _dev(d["v"][:, :, a:b]), 0.8)
        assert_cache_equal(oc, gc, f"rows {a}:{b}")


def test_quantize_reciprocal_ties_over_scale_values(orc):
    """Rows built so that the stored scale is a chosen binary16 value s (extrema -s and 2s, clip 1) and the other
    elements sit on multiples of s/4: x/s + zero then lands exactly on .5 ties up to the rounding of 1/s, so the
    code of such an element is decided by the last bit of the reciprocal.  Sweeps 3328 scale values (every eighth
    significand over 26 binades) through the un-rotated value path and compares codes and meta bit for bit."""
    sig = 1024 + 8 * np.arange(128)
    exps = np.arange(-12, 14)
    scales = (sig[None, :].astype(np.float64) * 2.0 ** (exps[:, None] - 10)).reshape(-1)
    T = scales.size
    assert T % 64 == 0
    rng = np.random.default_rng(5)
    mult = rng.integers(-4, 9, size=(T, 128)).astype(np.float64) / 4.0      # multiples of 1/4 in [-1, 2]
    mult[:, 0], mult[:, 1] = -1.0, 2.0
    mult[:, 2:8] = np.array([-0.5, 0.5, 1.5, -0.25, 0.75, 1.25])
    rows = (mult * scales[:, None]).astype(np.float16)
    assert np.array_equal(rows.astype(np.float64), mult * scales[:, None])   # all exactly representable
    v = rows[None, None]
    k = np.ascontiguousarray(v[:, :, ::-1])
    w = synth.small("ties", B=1, Hq=1, Hkv=1, T=T, G=128, clip=1.0)
    oc, gc = make_pair(orc, w, t_cap=T, s_cap=64)
    oc.quantize_append(k, v, 1.0, rotate_v=False)
    akvq.quantize_append(gc, _dev(k), _dev(v), 1.0, flags=akvq.V_PREROTATED)
    assert_cache_equal(oc, gc, "reciprocal ties")
    meta = oc.v_meta[0, 0, :T, 0]
    got_scale = (meta & 0x7FFF).astype(np.uint16).view(np.float16).astype(np.float64)
    assert np.array_equal(got_scale, scales)                                  # the sweep really hit every scale


def test_quantize_append_in_pieces_and_single_rows(orc):
    w = synth.small("pieces", B=1, Hq=2, Hkv=2, T=100, G=64)
    d = _np(synth.generate(w, seed=103))
    oc, gc = make_pair(orc, w, fill=0x5A, t_cap=128, s_cap=64)
    oc.select_psa(d["q_tail"], d["k"], 6, w.sm_scale)
    copy_salient_to_gpu(oc, gc)
    cuts = [0, 41, 42, 43, 64, 65, 97, 100]
    for a, b in zip(cuts[:-1], cuts[1:]):
        oc.quantize_append(d["k"][:, :, a:b], d["v"][:, :, a:b], 0.8)
        akvq.quantize_append(gc, _dev(d["k"][:, :, a:b]), _dev(d["v"][:, :, a:b]), 0.8)
        assert_cache_equal(oc, gc, f"rows {a}:{b}")


def test_quantize_prerotated_values(orc):
    w = synth.small("prerot", B=1, Hq=2, Hkv=2, T=64, G=128)
    d = _np(synth.generate(w, seed=104))
    oc, gc = make_pair(orc, w, t_cap=64, s_cap=64)
    oc.quantize_append(d["k"], d["v"], 0.8, rotate_v=False)
    akvq.quantize_append(gc, _dev(d["k"]), _dev(d["v"]), 0.8, flags=akvq.V_PREROTATED)
    assert_cache_equal(oc, gc, "prerotated V")


def test_quantize_adversarial_rows(orc):
    """Constant rows, exact ties, tiny and huge magnitudes, zero rows."""
    rng = np.random.default_rng(5)
    T = 64
    k = rng.standard_normal((1, 1, T, D)).astype(np.float16)
    k[0, 0, 0] = 0.0
    k[0, 0, 1] = 2.75
    k[0, 0, 2] = np.float16(6e-8)
    k[0, 0, 3] = 60000.0
    k[0, 0, 4, ::2] = 1.0; k[0, 0, 4, 1::2] = -1.0
    k[0, 0, 5] = (np.arange(D) % 4).astype(np.float16) - 1.5
    k[0, 0, 6] = (rng.integers(-8, 9, D) * 0.5).astype(np.float16)
    k[0, 0, 7] = np.where(np.arange(D) == 17, 1000.0, 1e-3).astype(np.float16)
    v = k[:, :, ::-1].copy()
    for G in (128, 64):
        for clip in (1.0, 0.8, 0.5):
            oc = orc.OracleCache(1, 1, G, 64, 64)
            gc = akvq.Cache(1, 1, G, 64, 64, fill=0)
            oc.quantize_append(k, v, clip)
            akvq.quantize_append(gc, _dev(k), _dev(v), clip)
            assert_cache_equal(oc, gc, f"adversarial G={G} clip={clip}")
            oc2 = orc.OracleCache(1, 1, G, 64, 64)
            gc2 = akvq.Cache(1, 1, G, 64, 64, fill=0)
            oc2.quantize_append(k, v, clip, rotate_v=False)
            akvq.quantize_append(gc2, _dev(k), _dev(v), clip, flags=akvq.V_PREROTATED)
            assert_cache_equal(oc2, gc2, f"adversarial prerotated G={G} clip={clip}")


# ------------------------------------------------------------------------------------------- selection
def test_select_tsa_exact(orc):
    w = synth.small("tsa", B=3, Hq=4, Hkv=2, T=700, n_text_head=37, n_text_tail=41)
    d = _np(synth.generate(w, seed=105))
    mask = d["is_text"].copy()
    mask[1, 100:400:7] = 1       # a batch element with scattered text
    mask[2] = 0                  # and one without any
    oc, gc = make_pair(orc, w, t_cap=704, s_cap=128)
    oc.select_tsa(mask)
    akvq.select_salient(gc, akvq.MODE_TSA, is_text=_dev(mask))
    torch.cuda.synchronize()
    assert np.array_equal(gc.counts().cpu().numpy(), oc.sal_cnt)
    for b in range(3):
        for h in range(2):
            n = min(oc.sal_cnt[b, h], 128)
            assert np.array_equal(gc.sal_idx[b, h, :n].cpu().numpy(), oc.sal_idx[b, h, :n])
    # capacity: more text than slots -> count reports the truth, first S_cap positions stored
    oc2, gc2 = make_pair(orc, w, t_cap=704, s_cap=64)
    oc2.select_tsa(mask)
    akvq.select_salient(gc2, akvq.MODE_TSA, is_text=_dev(mask))
    torch.cuda.synchronize()
    assert np.array_equal(gc2.counts().cpu().numpy(), oc2.sal_cnt) and oc2.sal_cnt.max() > 64
    assert np.array_equal(gc2.sal_idx.cpu().numpy()[:2], oc2.sal_idx[:2])


# Pivot index sets are compared EXACTLY.  What makes that well-posed: the inputs of every such comparison are accepted
# by psa_inputs.margin_checked only if the oracle's fp64 masses leave a relative gap of at least 1e-4 between the k-th
# and the (k+1)-th mass in every (batch, kv-head); the GPU's fp32 masses are held to MASS_RTOL of the oracle's, element
# by element, relative to the element itself (fp32 logits of magnitude up to ~2^8 in the base-2 domain carry an error
# of a few 2^-16 ulp-of-256 = 1.5e-5 each, which is the relative error of their exponentials; row sums and the final
# sums are far more exact), so a swap at the boundary would need an error above half the gap.
MASS_RTOL = 4e-5
MASS_ATOL = 1e-12


def check_psa(orc, w, seed, top_k, share_heads=False):
    d, seed, oc, mass_ref, margins = psa_inputs.margin_checked(orc, synth.generate, w, seed, top_k, share_heads)
    gc = akvq.Cache(w.B, w.Hkv, w.G, (w.T + 63) // 64 * 64, max(64, (top_k + 63) // 64 * 64))
    mass = torch.zeros(w.B, w.Hkv, w.T, dtype=torch.float32, device="cuda")
    akvq.select_salient(gc, akvq.MODE_PSA_SHARED if share_heads else akvq.MODE_PSA, q_tail=_dev(d["q_tail"]),
                        k=_dev(d["k"]), top_k=top_k, sm_scale=w.sm_scale, mass_out=mass)
    torch.cuda.synchronize()
    mass32 = mass.cpu().numpy()
    mass = mass32.astype(np.float64)
    assert np.allclose(mass.sum(-1), w.W * (w.Hq // w.Hkv), rtol=1e-5), "softmax rows must sum to one"
    err = np.abs(mass - mass_ref)
    worst = np.unravel_index(np.argmax(err - MASS_RTOL * mass_ref), err.shape)
    assert (err <= MASS_RTOL * mass_ref + MASS_ATOL).all(), \
        f"mass at {worst}: {mass[worst]:.9e} vs {mass_ref[worst]:.9e} (rel {err[worst] / mass_ref[worst]:.2e})"
    n = min(top_k, w.T)
    assert (gc.counts().cpu().numpy() == n).all()
    idx = gc.sal_idx.cpu().numpy()
    for b in range(w.B):
        total = None
        if share_heads:
            total = np.zeros(w.T, dtype=np.float32)
            for h in range(w.Hkv):
                total = total + mass32[b, h]                       # head order, fp32: what the kernel adds
        for h in range(w.Hkv):
            got, ref = idx[b, h, :n], oc.sal_idx[b, h, :n]
            assert (np.diff(got) > 0).all(), "indices must be ascending and distinct"
            # the GPU's own masses must make its set a correct top-k (ties to the lower position) ...
            gm = total if share_heads else mass32[b, h]
            order = sorted(range(w.T), key=lambda t: (-gm[t], t))[:n]
            assert sorted(order) == list(got), f"top-k of the GPU masses wrong at {(b, h)}"
            # ... and the set is the oracle's, exactly
            assert np.array_equal(got, ref), \
                f"{w.name} seed {seed}: salient set of {(b, h)} differs from the oracle's (margin " \
                f"{margins[b] if share_heads else margins[b, h]:.2e}): {sorted(set(got) ^ set(ref))}"
    big = mass_ref > 1e-6                                         # below that the absolute floor decides, not the ratio
    return float((err[big] / mass_ref[big]).max())


def test_select_psa_small(orc):
    w = synth.small("psa", B=2, Hq=4, Hkv=2, T=300, W=16, top_k=8)
    check_psa(orc, w, 106, 8)


@pytest.mark.parametrize("R,T", [(4, 2500), (5, 130), (6, 2049), (8, 4200), (2, 64)])
def test_select_psa_grouped_heads(orc, R, T):
    """W = 64 with several query heads per KV head: the kernels with a wavefront per head (a feeder wavefront below
    eight heads, shared loading with eight); contexts of one block, of a chunk plus one key, of several chunks."""
    w = synth.small(f"psa_gqa{R}", B=2, Hq=2 * R, Hkv=2, T=T, W=64, top_k=min(16, T), n_text_head=4, n_text_tail=1)
    check_psa(orc, w, 4100 + 10 * R, w.top_k)


def test_select_psa_longer_than_the_staged_topk(orc):
    """More than 32768 keys: 17 score chunks per head and the top-k that reads its keys from memory instead of LDS;
    top_k above the short-list limit takes the general ordering path as well."""
    w = synth.small("psa_long", B=1, Hq=2, Hkv=1, T=33111, W=16, top_k=12, n_text_head=40, n_text_tail=31)
    check_psa(orc, w, 161, 12)
    check_psa(orc, w, 161, 300)


def test_select_psa_cfg1(orc):
    """Config 1 (the parity configuration): every head's pivot set equals the oracle's."""
    w = synth.WORKLOADS["cfg1"]
    worst = check_psa(orc, w, synth.BASE_SEED, w.top_k)
    print(f"cfg1: worst relative mass error {worst:.2e}")
    # planted pivots attract the mass (Section III-A.3): all four are in every head's set
    d = _np(synth.generate(w))
    oc = orc.OracleCache(w.B, w.Hkv, w.G, 640, 64)
    oc.select_psa(d["q_tail"], d["k"], w.top_k, w.sm_scale)
    hits = [len(set(d["pivots"][0].tolist()) & set(oc.sal_idx[0, h, :w.top_k].tolist())) for h in range(w.Hkv)]
    assert min(hits) >= 3 and np.mean(hits) > 3.8


# ------------------------------------------------------------------------------------------- decode attention
def run_decode_case(orc, w, d, mode, top_k, n_splits=(0,), T=None, clip=0.8, flags=0, lse_tol=2e-3):
    T = T or w.T
    k, v = d["k"][:, :, :T], d["v"][:, :, :T]
    n_sal = T if mode == "all" else max(top_k, w.n_text)
    oc, gc = make_pair(orc, w, t_cap=(T + 63) // 64 * 64, s_cap=max(64, (n_sal + 63) // 64 * 64))
    if mode == "tsa":
        oc.select_tsa(d["is_text"][:, :T])
    elif mode == "psa":
        oc.select_psa(d["q_tail"], k, top_k, w.sm_scale)
    elif mode == "all":
        oc.select_tsa(np.ones((w.B, T), dtype=np.uint8))
    copy_salient_to_gpu(oc, gc)
    wflags = flags & (akvq.K_PREROTATED | akvq.V_PREROTATED)
    oc.quantize_append(k, v, clip, rotate_v=not (flags & akvq.V_PREROTATED), rotate_k=not (flags & akvq.K_PREROTATED))
    akvq.quantize_append(gc, _dev(k), _dev(v), clip, flags=wflags)
    assert_cache_equal(oc, gc, "decode case cache")
    out_ref, lse_ref = oc.decode(d["q"], w.sm_scale, unrotate=not (flags & akvq.OUT_ROTATED),
                                 rotate_q=not (flags & akvq.Q_PREROTATED))
    flags &= akvq.OUT_ROTATED | akvq.Q_PREROTATED
    q = _dev(d["q"])
    worst = 0.0
    for ns in n_splits:
        out, lse = akvq.decode_attention(gc, q, w.sm_scale, n_split=ns, flags=flags)
        torch.cuda.synchronize()
        worst = max(worst, assert_attention_close(out, lse, out_ref, lse_ref, f"{w.name} {mode} T={T} n_split={ns}",
                                                  lse_tol=lse_tol))
    return worst


@pytest.mark.parametrize("mode", ["tsa", "psa", "none", "all"])
@pytest.mark.parametrize("G", [128, 64])
def test_decode_mha_small(orc, mode, G):
    w = synth.small(f"dmha{G}", B=2, Hq=3, Hkv=3, T=200, G=G, n_text_head=20, n_text_tail=9, top_k=7, W=16)
    d = _np(synth.generate(w, seed=107))
    run_decode_case(orc, w, d, mode, 7, n_splits=(1, 2, 3))


@pytest.mark.parametrize("mode", ["tsa", "psa"])
def test_decode_mha_many_workgroups(orc, mode):
    """More (batch, head) units than the chip holds workgroups at once, with and without a KV split."""
    w = synth.small("dmha_wide", B=17, Hq=32, Hkv=32, T=150, G=128, n_text_head=11, n_text_tail=6, top_k=5, W=16)
    d = _np(synth.generate(w, seed=131))
    run_decode_case(orc, w, d, mode, 5, n_splits=(1, 2))


@pytest.mark.parametrize("T", [1, 2, 31, 33, 64, 65, 127, 129])
def test_decode_ragged_lengths(orc, T):
    w = synth.small("ragged", B=1, Hq=2, Hkv=2, T=140, G=128, n_text_head=3, n_text_tail=3, W=16)
    d = _np(synth.generate(w, seed=108))
    run_decode_case(orc, w, d, "tsa", 4, n_splits=(1, 2), T=T)


@pytest.mark.parametrize("Hq,Hkv,G", [(4, 2, 128), (14, 2, 64), (8, 1, 64), (3, 1, 128)])
@pytest.mark.parametrize("mode", ["tsa", "psa"])
def test_decode_gqa_small(orc, Hq, Hkv, G, mode):
    w = synth.small(f"dgqa{Hq}_{Hkv}", B=2, Hq=Hq, Hkv=Hkv, T=333, G=G, n_text_head=33, n_text_tail=12, top_k=9, W=16)
    d = _np(synth.generate(w, seed=109))
    run_decode_case(orc, w, d, mode, 9, n_splits=(1, 4, 5))


@pytest.mark.parametrize("Hq,Hkv,G", [(1, 1, 128), (7, 1, 64)])
def test_decode_long_context_small_batch(orc, Hq, Hkv, G):
    """33 thousand rows in one (batch, kv-head): more than a thousand tiles per workgroup without a split, and the
    default and a large split count."""
    w = synth.small(f"long{Hq}", B=1, Hq=Hq, Hkv=Hkv, T=33050, G=G, n_text_head=30, n_text_tail=21, top_k=5, W=16)
    d = _np(synth.generate(w, seed=163))
    run_decode_case(orc, w, d, "tsa", 5, n_splits=(1, 0, 37))


@pytest.mark.parametrize("Hq,Hkv,G", [(3, 3, 128), (14, 2, 64)])
def test_decode_fp16_output_flag(orc, Hq, Hkv, G):
    """AKVQ_OUT_FP16: the output is the fp32 result rounded to binary16 (bit for bit), with one split (stored by the
    attention kernel) and with several (stored by the merge kernel), also combined with a rotated output."""
    w = synth.small(f"half{Hq}", B=2, Hq=Hq, Hkv=Hkv, T=260, G=G, n_text_head=9, n_text_tail=5, top_k=6, W=16)
    d = _np(synth.generate(w, seed=231))
    oc, gc = make_pair(orc, w, t_cap=320, s_cap=64)
    oc.select_tsa(d["is_text"])
    copy_salient_to_gpu(oc, gc)
    oc.quantize_append(d["k"], d["v"], w.clip)
    akvq.quantize_append(gc, _dev(d["k"]), _dev(d["v"]), w.clip)
    q = _dev(d["q"])
    for flags in (0, akvq.OUT_ROTATED):
        ref, lse_ref = oc.decode(d["q"], w.sm_scale, unrotate=not flags)
        for ns in (1, 3):
            full, _ = akvq.decode_attention(gc, q, w.sm_scale, n_split=ns, flags=flags)
            half, lse = akvq.decode_attention(gc, q, w.sm_scale, n_split=ns, flags=flags | akvq.OUT_FP16)
            torch.cuda.synchronize()
            assert half.dtype == torch.float16 and torch.equal(half, full.half()), f"flags={flags} n_split={ns}"
            assert_attention_close(half.float(), lse, ref, lse_ref, f"fp16 output flags={flags} n_split={ns}")


def test_decode_rotated_output_flag(orc):
    w = synth.small("rotout", B=1, Hq=2, Hkv=2, T=100, W=16)
    d = _np(synth.generate(w, seed=110))
    run_decode_case(orc, w, d, "psa", 4, n_splits=(2,), flags=akvq.OUT_ROTATED)


@pytest.mark.parametrize("Hq,Hkv,G", [(3, 3, 128), (2, 2, 64), (6, 2, 128)])
def test_no_rotation_mode(orc, Hq, Hkv, G):
    """All four rotation flags: rows are quantized as they arrive, q and the output are used as given (plain
    round-to-nearest quantization, the ablation baseline of Table III)."""
    w = synth.small(f"norot{Hq}_{G}", B=2, Hq=Hq, Hkv=Hkv, T=170, G=G, n_text_head=9, n_text_tail=5, top_k=6, W=16)
    d = _np(synth.generate(w, seed=141))
    allf = akvq.K_PREROTATED | akvq.V_PREROTATED | akvq.Q_PREROTATED | akvq.OUT_ROTATED
    # An un-rotated query keeps its outlier channel, and one product then carries most of a logit (here up to 118 in
    # the base-e domain).  The grouped-query kernel stages queries as two bfloat16 terms (16 bits), so a logit, and with
    # it the log-sum-exp, can be off by 2^-16 of that product; the output bar is unchanged.
    lse_tol = 2e-3 if Hq == Hkv else 6e-3
    run_decode_case(orc, w, d, "tsa", 6, n_splits=(1, 3), flags=allf, lse_tol=lse_tol)
    run_decode_case(orc, w, d, "psa", 6, n_splits=(2,), flags=akvq.K_PREROTATED | akvq.Q_PREROTATED, lse_tol=lse_tol)
    # every row salient: the overlay rows come from the pass behind the block kernel, which must honour the flags too
    run_decode_case(orc, w, d, "all", 6, n_splits=(1,), flags=allf, lse_tol=lse_tol)
    run_decode_case(orc, w, d, "all", 6, n_splits=(2,), flags=akvq.V_PREROTATED, lse_tol=lse_tol)


@pytest.mark.parametrize("mode,clip", [("tsa", 0.8), ("psa", 0.8), ("tsa", 1.0), ("psa", 1.0)])
def test_cfg1_end_to_end(orc, mode, clip):
    """Config 1: one layer, 32 heads, 640 tokens (35 text + 576 vision + 29 text), both salient modes, whole path on
    the GPU: select -> quantize -> decode."""
    w = synth.WORKLOADS["cfg1"]
    if mode == "psa":   # the base seed passes the margin check (tests/golden/psa_seed_search.txt); searched again here
        d, _, _, _, _ = psa_inputs.margin_checked(orc, synth.generate, w, synth.BASE_SEED, w.top_k)
    else:
        d = _np(synth.generate(w))
    oc, gc = make_pair(orc, w)
    k, v, q, qt = _dev(d["k"]), _dev(d["v"]), _dev(d["q"]), _dev(d["q_tail"])
    if mode == "tsa":
        oc.select_tsa(d["is_text"])
        akvq.select_salient(gc, akvq.MODE_TSA, is_text=_dev(d["is_text"]))
    else:
        oc.select_psa(d["q_tail"], d["k"], w.top_k, w.sm_scale)
        akvq.select_salient(gc, akvq.MODE_PSA, q_tail=qt, k=k, top_k=w.top_k, sm_scale=w.sm_scale)
    torch.cuda.synchronize()
    n = w.top_k if mode == "psa" else 64
    assert np.array_equal(gc.counts().cpu().numpy(), oc.sal_cnt)
    assert np.array_equal(gc.sal_idx.cpu().numpy()[..., :n], oc.sal_idx[..., :n]), f"cfg1 {mode}: salient sets differ"
    oc.quantize_append(d["k"], d["v"], clip)
    akvq.quantize_append(gc, k, v, clip)
    assert_cache_equal(oc, gc, f"cfg1 {mode}")
    out_ref, lse_ref = oc.decode(d["q"], w.sm_scale)
    for ns in (0, 1, 5):
        out, lse = akvq.decode_attention(gc, q, w.sm_scale, n_split=ns)
        assert_attention_close(out, lse, out_ref, lse_ref, f"cfg1 {mode} n_split={ns}")


def test_decode_then_append_then_decode(orc):
    """Decode-phase use: one new row per step, some of them salient (listed by the caller)."""
    w = synth.small("steps", B=1, Hq=2, Hkv=2, T=90, W=16)
    d = _np(synth.generate(w, seed=111))
    oc, gc = make_pair(orc, w, t_cap=128, s_cap=64)
    oc.select_tsa(d["is_text"])               # tail text positions 87..89 arrive during decode and are salient
    copy_salient_to_gpu(oc, gc)
    oc.quantize_append(d["k"][:, :, :80], d["v"][:, :, :80], 0.8)
    akvq.quantize_append(gc, _dev(d["k"][:, :, :80]), _dev(d["v"][:, :, :80]), 0.8)
    for t in range(80, 90):
        oc.quantize_append(d["k"][:, :, t:t + 1], d["v"][:, :, t:t + 1], 0.8)
        akvq.quantize_append(gc, _dev(d["k"][:, :, t:t + 1]), _dev(d["v"][:, :, t:t + 1]), 0.8)
        out_ref, lse_ref = oc.decode(d["q"], w.sm_scale)
        out, lse = akvq.decode_attention(gc, _dev(d["q"]), w.sm_scale, n_split=2)
        assert_attention_close(out, lse, out_ref, lse_ref, f"step {t}")
    assert_cache_equal(oc, gc, "after decode steps")


@pytest.mark.parametrize("G,flags", [(128, 0), (64, 0), (128, akvq.V_PREROTATED), (64, akvq.K_PREROTATED | akvq.V_PREROTATED)])
def test_single_row_appends(orc, G, flags):
    """The decode step's append (one row per (batch, kv-head)) over 45 consecutive positions across block boundaries,
    some of the new rows listed as salient beforehand; the cache is compared bit for bit after every row."""
    w = synth.small(f"one{G}", B=2, Hq=3, Hkv=3, T=90, G=G, n_text_head=7, n_text_tail=4, top_k=5, W=16)
    d = _np(synth.generate(w, seed=151))
    T0 = 45
    oc, gc = make_pair(orc, w, t_cap=128, s_cap=64)
    listed = np.array([3, 17, 44, 45, 46, 63, 64, 70, 89], dtype=np.int32)     # rows before and after the prefill end
    oc.sal_idx[:, :, :len(listed)] = listed
    oc.sal_cnt[:] = len(listed)
    copy_salient_to_gpu(oc, gc)
    rk, rv = not (flags & akvq.K_PREROTATED), not (flags & akvq.V_PREROTATED)
    oc.quantize_append(d["k"][:, :, :T0], d["v"][:, :, :T0], w.clip, rotate_v=rv, rotate_k=rk)
    akvq.quantize_append(gc, _dev(d["k"][:, :, :T0]), _dev(d["v"][:, :, :T0]), w.clip, flags=flags)
    for t in range(T0, w.T):
        k1, v1 = d["k"][:, :, t:t + 1], d["v"][:, :, t:t + 1]
        oc.quantize_append(k1, v1, w.clip, rotate_v=rv, rotate_k=rk)
        akvq.quantize_append(gc, _dev(k1), _dev(v1), w.clip, flags=flags)
        assert_cache_equal(oc, gc, f"after row {t}")


# ------------------------------------------------------------------------------------------- error paths (no launch)
def test_argument_errors():
    L = akvq.lib()
    gc = akvq.Cache(1, 2, 128, 64, 64)
    q = torch.zeros(1, 2, D, dtype=torch.float16, device="cuda")
    with pytest.raises(akvq.AkvqError, match="invalid argument"):
        akvq.decode_attention(gc, q, 0.1)                    # T_len == 0
    k = torch.zeros(1, 2, 65, D, dtype=torch.float16, device="cuda")
    with pytest.raises(akvq.AkvqError, match="capacity"):
        akvq.quantize_append(gc, k, k, 0.8)                  # 65 rows into T_cap 64
    with pytest.raises(akvq.AkvqError, match="invalid argument"):
        akvq.quantize_append(gc, k[:, :, :4].contiguous(), k[:, :, :4].contiguous(), 1.5)   # clip out of (0,1]
    bad = akvq.akvq_cache(1, 2, 96, 64, 64, 0)
    import ctypes as C
    sizes = (C.c_size_t * 8)()
    assert L.akvq_cache_bytes(C.byref(bad), sizes) == -2     # unsupported group size
    qt = torch.zeros(1, 4, 24, D, dtype=torch.float16, device="cuda")
    kk = torch.zeros(1, 2, 64, D, dtype=torch.float16, device="cuda")
    with pytest.raises(akvq.AkvqError, match="unsupported"):
        akvq.select_salient(gc, akvq.MODE_PSA, q_tail=qt, k=kk, top_k=4, sm_scale=0.1)      # W not a multiple of 16
    qt = torch.zeros(1, 4, 16, D, dtype=torch.float16, device="cuda")
    with pytest.raises(akvq.AkvqError, match="capacity"):
        akvq.select_salient(gc, akvq.MODE_PSA, q_tail=qt, k=kk, top_k=65, sm_scale=0.1)     # top_k > S_cap


def test_results_do_not_depend_on_the_run():
    """The same inputs twice (fresh caches, other work in between): index sets, cache bytes, masses and attention
    outputs are bit-identical -- no result depends on the order in which workgroups or atomics happen to run."""
    w = synth.small("det", B=3, Hq=14, Hkv=2, T=2300, G=64, n_text_head=40, n_text_tail=25, top_k=24, W=32)
    d = synth.generate(w, seed=201, device="cuda")
    runs = []
    for rep in range(2):
        c = akvq.Cache(w.B, w.Hkv, w.G, 2304, 64, fill=0)
        c.enable_window(64)
        mass = torch.zeros(w.B, w.Hkv, w.T, device="cuda")
        akvq.select_salient(c, akvq.MODE_PSA, q_tail=d["q_tail"], k=d["k"], top_k=w.top_k, sm_scale=w.sm_scale,
                            mass_out=mass)
        akvq.quantize_append_tiered(c, d["k"], d["v"], None, None, w.clip, 1.0)
        out, lse = akvq.decode_attention(c, d["q"], w.sm_scale, n_split=5)
        torch.cuda.synchronize()
        runs.append([t.clone() for t in (mass, c.sal_idx, c.k_codes, c.v_codes, c.k_meta, c.v_meta, c.k_sal, c.v_sal,
                                         c.k_win, c.v_win, out, lse)])
        torch.randn(1 << 22, device="cuda").sort()          # unrelated work between the two runs
    for a, b in zip(*runs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (8, 2)])
@pytest.mark.parametrize("sm_scale", [0.0, 1.0, -0.05, 1e-4])
def test_decode_softmax_scales(orc, Hq, Hkv, sm_scale):
    """Flat (scale 0: the plain mean of the value rows), very peaked, and negated logits."""
    w = synth.small(f"scale{Hq}", B=2, Hq=Hq, Hkv=Hkv, T=210, G=128, n_text_head=9, n_text_tail=5, top_k=5, W=16)
    d = _np(synth.generate(w, seed=171))
    oc, gc = make_pair(orc, w, t_cap=256, s_cap=64)
    oc.select_tsa(d["is_text"])
    copy_salient_to_gpu(oc, gc)
    oc.quantize_append(d["k"], d["v"], w.clip)
    akvq.quantize_append(gc, _dev(d["k"]), _dev(d["v"]), w.clip)
    ref, lse_ref = oc.decode(d["q"], sm_scale)
    for ns in (1, 3):
        out, lse = akvq.decode_attention(gc, _dev(d["q"]), sm_scale, n_split=ns)
        torch.cuda.synchronize()
        # logits reach the hundreds at scale 1: the log-sum-exp can only be as exact as fp32 and the two-term queries
        # of the grouped-query kernel are at that magnitude (the output bar is unchanged)
        assert_attention_close(out, lse, ref, lse_ref, f"sm_scale={sm_scale} n_split={ns}",
                               lse_tol=max(2e-3, 5e-5 * float(np.abs(lse_ref).max())))


@pytest.mark.parametrize("Hq,Hkv", [(3, 3), (8, 2)])
def test_non_finite_inputs_stay_in_their_unit(orc, Hq, Hkv):
    """NaN and infinities in the rows of one (batch, kv-head): its results are unspecified, nothing faults, and every
    other unit is exactly what it is without them (selection, cache bytes, attention)."""
    w = synth.small(f"nonfinite{Hq}", B=2, Hq=Hq, Hkv=Hkv, T=200, G=128, n_text_head=9, n_text_tail=5, top_k=6, W=16)
    d = _np(synth.generate(w, seed=211))
    k, v = d["k"].copy(), d["v"].copy()
    k[0, 0, 5, :] = np.nan
    k[0, 0, 9, 0] = -np.inf
    v[0, 0, 7, 3] = np.inf
    v[0, 0, 150, 64:] = np.nan
    oc, gc = make_pair(orc, w, t_cap=256, s_cap=64)
    clean = orc.OracleCache(w.B, w.Hkv, w.G, 256, 64, fill=0)
    clean.select_psa(d["q_tail"], d["k"], w.top_k, w.sm_scale)
    clean.quantize_append(d["k"], d["v"], w.clip)
    ref, lse_ref = clean.decode(d["q"], w.sm_scale)
    akvq.select_salient(gc, akvq.MODE_PSA, q_tail=_dev(d["q_tail"]), k=_dev(k), top_k=w.top_k, sm_scale=w.sm_scale)
    akvq.quantize_append(gc, _dev(k), _dev(v), w.clip)
    out, lse = akvq.decode_attention(gc, _dev(d["q"]), w.sm_scale, n_split=2)
    torch.cuda.synchronize()
    R = Hq // Hkv
    for b in range(w.B):
        for h in range(Hkv):
            if (b, h) == (0, 0):
                continue
            n = int(clean.sal_cnt[b, h])
            assert int(gc.counts()[b, h]) == n
            assert np.array_equal(gc.sal_idx[b, h, :n].cpu().numpy(), clean.sal_idx[b, h, :n])
            for name in ("k_codes", "v_codes", "k_meta", "v_meta"):
                got = _u32(getattr(gc, name)[b, h])
                assert np.array_equal(got, getattr(clean, name)[b, h]), (name, b, h)
            heads = slice(h * R, (h + 1) * R)
            assert_attention_close(out[b:b + 1, heads], lse[b:b + 1, heads], ref[b:b + 1, heads], lse_ref[b:b + 1, heads],
                                   f"unit {(b, h)}")


@pytest.mark.parametrize("Hq,Hkv,T,top_k", [(6, 3, 500, 7), (8, 8, 2100, 16), (14, 2, 333, 4)])
def test_select_psa_token_level(orc, Hq, Hkv, T, top_k):
    """AKVQ_MODE_PSA_SHARED: the kv-heads' masses are added and every head of a batch element gets the same list."""
    w = synth.small(f"psa_sh{Hq}", B=2, Hq=Hq, Hkv=Hkv, T=T, W=16, top_k=top_k, n_text_head=9, n_text_tail=4)
    check_psa(orc, w, 221, top_k, share_heads=True)
