"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (default KV splits).

The HIP path runs on the whole workload; a few (batch, kv-head) units are then copied to the host and the oracle
recomputes exactly those units from the same inputs: salient sets equal (exactly; the inputs pass the margin check of
psa_inputs on those units), codes / meta / overlay rows bit-exact, attention within the stated tolerance.  Inputs are drawn on the GPU with the seeded generator (the oracle sees the very
same bits).
"""
import numpy as np
import pytest
import torch

import psa_inputs
from paper_2501_15021_amd import binding as akvq
from paper_2501_15021_amd import synth

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3  # per (b, hq): max_d |o_gpu - o_ref| <= 2e-3 * max_d |o_ref|


def _unit_cache(orc, w, layer):
    return orc.OracleCache(1, 1, w.G, (w.T + 63) // 64 * 64, w.s_cap(layer))


def _unit_selection(orc, w, layer, d, b, h):
    """The oracle's salient list of one (batch, kv-head) unit from the same inputs, and (pivot layers) the fp64 margin
    (m_k - m_{k+1}) / m_k of its masses at the selection boundary."""
    R = w.Hq // w.Hkv
    oc = _unit_cache(orc, w, layer)
    if w.mode(layer) == "tsa":
        oc.select_tsa(d["is_text"][b:b + 1].cpu().numpy())
        return oc, np.inf
    k = d["k"][b:b + 1, h:h + 1].cpu().numpy()
    mass = oc.select_psa(d["q_tail"][b:b + 1, h * R:(h + 1) * R].cpu().numpy(), k, w.top_k, w.sm_scale, want_mass=True)
    return oc, float(orc.topk_margins(mass, w.top_k)[0, 0])


def _margin_checked_inputs(orc, w, layer, units):
    """Full-size inputs are drawn on the GPU, so the seed search of the index-set protocol runs here, over the sampled
    units (the ones that are compared): a seed is accepted when each of them has an fp64 margin of at least 1e-4."""
    for seed in range(synth.BASE_SEED, synth.BASE_SEED + psa_inputs.MAX_TRIES):
        d = synth.generate(w, seed=seed, layer=layer, device="cuda")
        sel = {u: _unit_selection(orc, w, layer, d, *u) for u in units}
        m = np.array([sel[u][1] for u in units])
        ok = bool((m >= psa_inputs.MIN_MARGIN).all())
        tight = [f"{u} {x:.2e}" for u, x in zip(units, m) if x < psa_inputs.REPORT_MARGIN]
        print(f"psa seed search [{w.name} layer {layer}, sampled units {units}]: seed {seed}: min margin {m.min():.3e}"
              + (f", below {psa_inputs.REPORT_MARGIN:g}: {', '.join(tight)}" if tight else "")
              + (": accepted" if ok else ": rejected"), flush=True)
        if ok:
            return d, sel
    raise AssertionError("no seed passes the margin check")


def _check_units(orc, w, layer, d, cache, out_gpu, units, sel):
    R = w.Hq // w.Hkv
    t_cap = (w.T + 63) // 64 * 64
    n_blocks = t_cap // 32
    for (b, h) in units:
        print(f"unit b={b} kv-head={h}", flush=True)
        k = d["k"][b:b + 1, h:h + 1].cpu().numpy()
        v = d["v"][b:b + 1, h:h + 1].cpu().numpy()
        heads = slice(h * R, (h + 1) * R)
        oc, margin = sel[(b, h)]
        cnt = int(oc.sal_cnt[0, 0])
        assert int(cache.counts()[b, h]) == cnt
        got_idx = cache.sal_idx[b, h].cpu().numpy()
        assert np.array_equal(got_idx[:cnt], oc.sal_idx[0, 0, :cnt]), \
            f"salient set differs at unit {(b, h)} (margin {margin:.2e}): " \
            f"{sorted(set(got_idx[:cnt].tolist()) ^ set(oc.sal_idx[0, 0, :cnt].tolist()))}"
        oc.quantize_append(k, v, w.clip)
        for name in ("k_codes", "v_codes"):
            got = getattr(cache, name)[b, h].cpu().numpy().view(np.uint32).reshape(-1)
            ref = getattr(oc, name)[0, 0].reshape(-1)
            assert np.array_equal(got[:n_blocks * 256], ref[:n_blocks * 256]), f"{name} differ at unit {(b, h)}"
        for name in ("k_meta", "v_meta"):
            got = getattr(cache, name)[b, h].cpu().numpy().view(np.uint32)[:w.T].reshape(-1)
            assert np.array_equal(got, getattr(oc, name)[0, 0, :w.T].reshape(-1)), f"{name} differ at unit {(b, h)}"
        for name in ("k_sal", "v_sal"):
            got = getattr(cache, name)[b, h].cpu().numpy().view(np.uint16).reshape(-1)
            assert np.array_equal(got, getattr(oc, name)[0, 0].reshape(-1)), f"{name} differ at unit {(b, h)}"
        ref, _ = oc.decode(d["q"][b:b + 1, heads].cpu().numpy(), w.sm_scale)
        got = out_gpu[b, heads].cpu().numpy().astype(np.float64)
        err = np.abs(got - ref[0]).max(axis=-1)
        scale = np.maximum(np.abs(ref[0]).max(axis=-1), 1e-6)
        assert (err / scale).max() <= ATTN_TOL, f"attention at unit {(b, h)}: {(err / scale).max():.3e}"


def _run(orc, name, layer, units):
    w = synth.WORKLOADS[name]
    d, sel = _margin_checked_inputs(orc, w, layer, units)
    cache = akvq.Cache(w.B, w.Hkv, w.G, (w.T + 63) // 64 * 64, w.s_cap(layer))
    if w.mode(layer) == "tsa":
        akvq.select_salient(cache, akvq.MODE_TSA, is_text=d["is_text"])
    else:
        akvq.select_salient(cache, akvq.MODE_PSA, q_tail=d["q_tail"], k=d["k"], top_k=w.top_k, sm_scale=w.sm_scale)
    akvq.quantize_append(cache, d["k"], d["v"], w.clip)
    out, _ = akvq.decode_attention(cache, d["q"], w.sm_scale)  # default split heuristic, as in bench.py
    torch.cuda.synchronize()
    _check_units(orc, w, layer, d, cache, out, units, sel)


def test_cfg2_text_salient_layer(orc):
    _run(orc, "cfg2", 0, [(0, 0), (15, 31)])


def test_cfg2_pivot_salient_layer(orc):
    _run(orc, "cfg2", 2, [(0, 0), (7, 13), (15, 31)])


def test_cfg3(orc):
    _run(orc, "cfg3", 0, [(0, 0), (63, 31)])


def test_cfg4(orc):
    _run(orc, "cfg4", 0, [(0, 0), (7, 31)])


def test_cfg5_gqa(orc):
    _run(orc, "cfg5", 0, [(0, 0), (31, 3)])


# --------------------------------------------------------------- 4-bit text tier + recent window at full size
def _run_tiered(orc, name, layer, units, W):
    """Section III-C.1 tiers at the benchmark's size: text tokens 4-bit (row pairs) except position 0, the pivots of
    the GPU's own selection 16-bit, the last W rows in the 16-bit window; sampled (batch, kv-head) units are recomputed
    by the oracle from the same inputs and the same salient rows."""
    w = synth.WORKLOADS[name]
    d = synth.generate(w, layer=layer, device="cuda")
    mask = d["is_text"].cpu().numpy()
    row_src, row_tier, row_of = synth.tiered_rows(mask, [[0]] * w.B)
    n_rows = row_src.shape[1]
    t_cap = (n_rows + 63) // 64 * 64
    cache = akvq.Cache(w.B, w.Hkv, w.G, t_cap, 64, fill=0)
    cache.enable_window(W)
    akvq.select_salient(cache, akvq.MODE_PSA, q_tail=d["q_tail"], k=d["k"], top_k=w.top_k, sm_scale=w.sm_scale)
    # token positions -> cache rows; tokens stored 4-bit are dropped from the list (ascending order is kept)
    idx = cache.sal_idx.cpu().numpy()
    cnt = cache.counts().cpu().numpy()
    plain = (mask == 0) | (np.arange(w.T)[None, :] == 0)
    new_idx = np.full_like(idx, -1)
    new_cnt = np.zeros_like(cnt)
    for b in range(w.B):
        for h in range(w.Hkv):
            rows = [int(row_of[b, t]) for t in idx[b, h, :cnt[b, h]] if plain[b, t]]
            new_idx[b, h, :len(rows)] = rows
            new_cnt[b, h] = len(rows)
    cache.sal_idx.copy_(torch.from_numpy(new_idx).cuda())
    cache.counts().copy_(torch.from_numpy(new_cnt).cuda())
    akvq.quantize_append_tiered(cache, d["k"], d["v"], torch.from_numpy(row_src).cuda(),
                                torch.from_numpy(row_tier).cuda(), w.clip, 1.0)
    out, _ = akvq.decode_attention(cache, d["q"], w.sm_scale)
    torch.cuda.synchronize()
    R = w.Hq // w.Hkv
    for (b, h) in units:
        print(f"tiered unit b={b} kv-head={h}", flush=True)
        oc = orc.OracleCache(1, 1, w.G, t_cap, 64, fill=0)
        oc.enable_window(W)
        n = int(new_cnt[b, h])
        oc.sal_idx[0, 0, :n] = new_idx[b, h, :n]
        oc.sal_cnt[0, 0] = n
        oc.quantize_append_tiered(d["k"][b:b + 1, h:h + 1].cpu().numpy(), d["v"][b:b + 1, h:h + 1].cpu().numpy(),
                                  row_src[b:b + 1], row_tier[b:b + 1], w.clip, 1.0)
        nb = (n_rows + 31) // 32
        for nm in ("k_codes", "v_codes"):
            got = getattr(cache, nm)[b, h].cpu().numpy().view(np.uint32)[:nb]
            assert np.array_equal(got, getattr(oc, nm)[0, 0, :nb]), f"{nm} differ at unit {(b, h)}"
        for nm in ("k_meta", "v_meta"):
            got = getattr(cache, nm)[b, h].cpu().numpy().view(np.uint32)[:n_rows]
            assert np.array_equal(got, getattr(oc, nm)[0, 0, :n_rows]), f"{nm} differ at unit {(b, h)}"
        for nm in ("k_sal", "v_sal", "k_win", "v_win"):
            got = getattr(cache, nm)[b, h].cpu().numpy().view(np.uint16).reshape(-1)
            assert np.array_equal(got, getattr(oc, nm)[0, 0].reshape(-1)), f"{nm} differ at unit {(b, h)}"
        assert np.array_equal(cache.fine_mask[b].cpu().numpy().view(np.uint32)[:nb], oc.fine_mask[0, :nb])
        heads = slice(h * R, (h + 1) * R)
        ref, _ = oc.decode(d["q"][b:b + 1, heads].cpu().numpy(), w.sm_scale)
        got = out[b, heads].cpu().numpy().astype(np.float64)
        err = np.abs(got - ref[0]).max(axis=-1)
        scale = np.maximum(np.abs(ref[0]).max(axis=-1), 1e-6)
        assert (err / scale).max() <= ATTN_TOL, f"tiered attention at unit {(b, h)}: {(err / scale).max():.3e}"


def test_cfg2_tiered_window(orc):
    _run_tiered(orc, "cfg2", 2, [(0, 0), (7, 13), (15, 31)], W=128)


def test_cfg5_tiered_window_gqa(orc):
    _run_tiered(orc, "cfg5", 0, [(0, 0), (31, 3)], W=128)


@pytest.mark.parametrize("Hq,G", [(8, 128), (16, 64)])
def test_planes_larger_than_4_gib(Hq, G):
    """Addressing beyond 32 bits: code planes of 4.8 GB each (300 x 8 kv-heads x 65536 rows).  64 rows are appended at
    the end of the last batch elements' planes and decode runs over the whole length; a one-sequence cache holding the
    same rows must give the same words and, with the same split, the same output bits."""
    B, Hkv, T_cap = 300, 8, 65536
    T0, n_new = T_cap - 64, 64
    big = akvq.Cache(B, Hkv, G, T_cap, 64, fill=0)
    assert big.k_codes.numel() * 4 > (1 << 32)
    g = torch.Generator(device="cuda").manual_seed(5)
    k = torch.randn(B, Hkv, n_new, 128, generator=g, device="cuda").half()
    v = torch.randn(B, Hkv, n_new, 128, generator=g, device="cuda").half()
    q = torch.randn(B, Hq, 128, generator=g, device="cuda").half()
    big.T_len = T0
    big.sal_idx[:, :, 0] = T0 + 3                       # one of the new rows is kept 16-bit
    big.counts().fill_(1)
    akvq.quantize_append(big, k, v, 0.8)
    out_big, lse_big = akvq.decode_attention(big, q, 0.0884, n_split=8)
    torch.cuda.synchronize()
    for b in (0, B - 1):
        small = akvq.Cache(1, Hkv, G, T_cap, 64, fill=0)
        small.T_len = T0
        small.sal_idx[:, :, 0] = T0 + 3
        small.counts().fill_(1)
        akvq.quantize_append(small, k[b:b + 1].contiguous(), v[b:b + 1].contiguous(), 0.8)
        out, lse = akvq.decode_attention(small, q[b:b + 1].contiguous(), 0.0884, n_split=8)
        torch.cuda.synchronize()
        for name in ("k_codes", "v_codes", "k_meta", "v_meta", "k_sal", "v_sal"):
            assert torch.equal(getattr(big, name)[b], getattr(small, name)[0]), f"{name} of batch element {b}"
        assert int(big.k_codes[b, -1, -2:].ne(0).sum()) > 0                # the appended blocks were written
        assert torch.equal(out_big[b], out[0]) and torch.equal(lse_big[b], lse[0]), f"decode of batch element {b}"
