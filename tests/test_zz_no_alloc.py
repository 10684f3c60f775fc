"""akvq_decode_attention_static (split-KV partials in the library's fixed device array, nothing allocated) against
akvq_decode_attention on the same cache: two calls in a row, the second on a smaller input, which must not be disturbed
by what the first left in the array.  Collected last: it shares one device array with every earlier call of its kind."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2501_15021_amd import binding as akvq
from paper_2501_15021_amd import synth

pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3


def _filled_cache(w, seed):
    d = synth.generate(w, seed=seed, device="cuda")
    c = akvq.Cache(w.B, w.Hkv, w.G, (w.T + 63) // 64 * 64, 64, fill=0)
    akvq.select_salient(c, akvq.MODE_PSA, q_tail=d["q_tail"], k=d["k"], top_k=w.top_k, sm_scale=w.sm_scale)
    akvq.quantize_append(c, d["k"], d["v"], w.clip)
    return c, d["q"]


@pytest.mark.parametrize("Hq,Hkv,G", [(6, 6, 128), (14, 2, 64)])
def test_static_scratch_matches_workspace_entry_point(Hq, Hkv, G):
    big = synth.small(f"noalloc_big{Hq}", B=3, Hq=Hq, Hkv=Hkv, T=1500, G=G, n_text_head=20, n_text_tail=9, top_k=12, W=16)
    small = synth.small(f"noalloc_small{Hq}", B=1, Hq=Hq, Hkv=Hkv, T=333, G=G, n_text_head=7, n_text_tail=5, top_k=5, W=16)
    cases = []
    for w, seed, ns in ((big, 301, 7), (small, 302, 3)):
        c, q = _filled_cache(w, seed)
        ref, lse_ref = akvq.decode_attention(c, q, w.sm_scale, n_split=ns)      # the existing entry point, caller workspace
        one, _ = akvq.decode_attention(c, q, w.sm_scale, n_split=1)             # no partials at all, for the 2e-3 bar
        out = torch.full_like(ref, float("nan"))
        lse = torch.full_like(lse_ref, float("nan"))
        cases.append((w, c, q, ns, ref, lse_ref, one, out, lse))
    torch.cuda.synchronize()
    for w, c, q, ns, ref, lse_ref, one, out, lse in cases:                      # back to back, the second one smaller
        akvq.decode_attention_static(c, q, w.sm_scale, out, lse, n_split=ns)
    torch.cuda.synchronize()
    for w, c, q, ns, ref, lse_ref, one, out, lse in cases:
        assert torch.equal(out, ref) and torch.equal(lse, lse_ref), f"{w.name}: differs from akvq_decode_attention"
        rel = (out - one).abs().amax(-1) / one.abs().amax(-1).clamp_min(1e-6)
        assert float(rel.max()) <= ATTN_TOL, f"{w.name}: {float(rel.max()):.3e} against the unsplit result"


def test_static_scratch_rejects_what_does_not_fit():
    """B * Hq * n_split partial slots beyond the 8 MiB array: AKVQ_ERR_WORKSPACE on the host, nothing launched."""
    L = akvq.lib()
    limit = L.akvq_decode_static_scratch_bytes()
    assert limit == 8 << 20
    c = akvq.Cache(2, 4, 128, 128, 64, fill=0)
    c.T_len = 100
    q = torch.zeros(2, 4, 128, dtype=torch.float16, device="cuda")
    out = torch.zeros(2, 4, 128, dtype=torch.float32, device="cuda")
    lse = torch.zeros(2, 4, dtype=torch.float32, device="cuda")
    assert L.akvq_decode_workspace_bytes(2, 4, 1024) <= limit
    big = akvq.Cache(32, 32, 128, 128, 64, fill=0)
    big.T_len = 100
    qb = torch.zeros(32, 32, 128, dtype=torch.float16, device="cuda")
    ob = torch.zeros(32, 32, 128, dtype=torch.float32, device="cuda")
    lb = torch.zeros(32, 32, dtype=torch.float32, device="cuda")
    assert L.akvq_decode_workspace_bytes(32, 32, 16) > limit
    with pytest.raises(akvq.AkvqError, match="workspace"):
        akvq.decode_attention_static(big, qb, 0.1, ob, lb, n_split=16)
    s = big.struct()
    assert L.akvq_decode_attention_static(C.byref(s), None, 32, 0.1, None, None, 16, 0, None) == -4   # size is checked first
    akvq.decode_attention_static(c, q, 0.1, out, lse, n_split=2)                 # a fitting call still works afterwards
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
