"""The library allocates nothing, synchronises nothing and records no memset: a decode step (append one row with the
rotary embedding fused in, then decode attention) can be captured in a HIP graph.  Every replay is checked against the
eager result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2501_15021_amd import binding as akvq
from paper_2501_15021_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("Hq,Hkv,G", [(4, 4, 128), (14, 2, 64)])
def test_decode_step_in_a_graph(Hq, Hkv, G):
    w = synth.small(f"graph{Hq}", B=3, Hq=Hq, Hkv=Hkv, T=200, G=G, n_text_head=12, n_text_tail=7, top_k=6, W=16)
    d = synth.generate(w, seed=181, device="cuda")
    T0 = w.T - 1
    cos, sin = (torch.from_numpy(t).cuda() for t in synth.rope_tables(np.arange(w.T)))
    new_rope = (cos[T0:].contiguous(), sin[T0:].contiguous())

    def fresh_cache():
        c = akvq.Cache(w.B, w.Hkv, G, 256, 64, fill=0)
        c.enable_window(64)
        akvq.select_salient(c, akvq.MODE_TSA, is_text=d["is_text"])
        akvq.quantize_append_tiered(c, d["k"][:, :, :T0].contiguous(), d["v"][:, :, :T0].contiguous(), None, None,
                                    w.clip, 1.0, rope=(cos[:T0].contiguous(), sin[:T0].contiguous()))
        return c

    k1, v1 = d["k"][:, :, T0:].contiguous(), d["v"][:, :, T0:].contiguous()
    out = torch.zeros(w.B, Hq, 128, device="cuda")
    lse = torch.zeros(w.B, Hq, device="cuda")

    def step(c):
        c.T_len = T0
        akvq.quantize_append_tiered(c, k1, v1, None, None, w.clip, 1.0, rope=new_rope)
        akvq.decode_attention(c, d["q"], w.sm_scale, n_split=3, out=out, lse=lse, rope=new_rope)

    eager_cache = fresh_cache()
    step(eager_cache)
    torch.cuda.synchronize()
    want_out, want_lse = out.clone(), lse.clone()

    cache = fresh_cache()
    step(cache)                              # warm-up on the capture cache: workspaces exist before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(cache)
    torch.cuda.synchronize()
    for replay in range(4):
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        cache.k_win[:, :, T0 % 64].zero_()   # eager work that undoes part of the step: the replay has to redo it
        cache.k_meta[:, :, T0].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want_out), f"replay {replay}: output differs from the eager step"
        assert torch.equal(lse, want_lse), f"replay {replay}"
        for name in ("k_codes", "v_codes", "k_meta", "v_meta", "k_win", "v_win", "k_sal", "v_sal"):
            assert torch.equal(getattr(cache, name), getattr(eager_cache, name)), f"replay {replay}: {name}"
