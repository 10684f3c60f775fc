"""Seeded synthetic inputs shaped like the paper's multimodal decode workloads.

This module only draws random inputs (it holds none of the method's arithmetic) and serves both the
GPU library and the CPU checker.  The paper evaluates on LLaVA-v1.5-7B with multi-image prompts
(Section IV-A); those prompts and weights are not available here, so the tensors below stand in
for them: 576 vision tokens per image (LLaVA-1.5's patch count), text segments around the images,
Keys with a few large-magnitude channels (the outlier pattern of Section III-C.2 / Fig. 5) and a few
high-norm pivot tokens (the pattern of Section III-A.3), layer split TSA 0-1 / PSA 2-31 (Table I).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np
import torch

D = 128
BASE_SEED = 250115021
N_OUTLIER_CHANNELS = 4
OUTLIER_GAIN = 20.0
N_PIVOTS = 4
PIVOT_GAIN = 10.0


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    T: int
    G: int
    segments: Tuple[Tuple[str, int], ...]   # ("text"|"vision", length) in prompt order
    top_k: int                              # pivots kept in PSA layers
    n_layers: int = 1
    tsa_layers: Tuple[int, ...] = ()        # layers whose salient set is the text tokens
    W: int = 64                             # query rows used for the pivot score
    clip: float = 0.8                       # Section IV-C: clip ratio 0.8 for 2-bit

    @property
    def sm_scale(self) -> float:
        return 1.0 / float(np.sqrt(D))

    @property
    def n_text(self) -> int:
        return sum(n for kind, n in self.segments if kind == "text")

    def mode(self, layer: int) -> str:
        return "tsa" if layer in self.tsa_layers else "psa"

    def s_cap(self, layer: int) -> int:
        n = self.n_text if self.mode(layer) == "tsa" else self.top_k
        return max(64, (n + 63) // 64 * 64)


def _interleave(first: int, gap: int, last: int, n_img: int):
    seg: List[Tuple[str, int]] = [("text", first)]
    for i in range(n_img):
        seg.append(("vision", 576))
        if i < n_img - 1 and gap:
            seg.append(("text", gap))
    seg.append(("text", last))
    return tuple(seg)


WORKLOADS = {
    # single layer, both modes are exercised by the tests (TSA keeps the 64 text rows, PSA keeps top-8)
    "cfg1": Workload("cfg1", B=1, Hq=32, Hkv=32, T=640, G=128,
                     segments=(("text", 35), ("vision", 576), ("text", 29)), top_k=8),
    # LLaVA-1.5-7B-shaped decode: 6 images, 640 interleaved text tokens, layers 0-1 TSA, 2-31 PSA top-16
    "cfg2": Workload("cfg2", B=16, Hq=32, Hkv=32, T=4096, G=128, segments=_interleave(100, 88, 100, 6),
                     top_k=16, n_layers=32, tsa_layers=(0, 1)),
    # long-video decode, per layer: 14 frames + 128 text, PSA top-32
    "cfg3": Workload("cfg3", B=64, Hq=32, Hkv=32, T=8192, G=128, segments=_interleave(64, 0, 64, 14), top_k=32),
    # prefill write path: 28 frames + 256 text, PSA top-32 from the last 64 rows
    "cfg4": Workload("cfg4", B=8, Hq=32, Hkv=32, T=16384, G=128, segments=_interleave(128, 0, 128, 28), top_k=32),
    # GQA 28/4, group 64, 56 frames + 512 text, PSA top-64
    "cfg5": Workload("cfg5", B=32, Hq=28, Hkv=4, T=32768, G=64, segments=_interleave(256, 0, 256, 56), top_k=64),
}
for _w in WORKLOADS.values():
    assert sum(n for _, n in _w.segments) == _w.T, _w.name


def is_text_mask(w: Workload) -> np.ndarray:
    """uint8 [T]: 1 where the prompt position holds a text token."""
    m = np.zeros(w.T, dtype=np.uint8)
    pos = 0
    for kind, n in w.segments:
        if kind == "text":
            m[pos:pos + n] = 1
        pos += n
    return m


def small(name: str, B: int, Hq: int, Hkv: int, T: int, G: int = 128, n_text_head: int = 5, n_text_tail: int = 3,
          top_k: int = 4, W: int = 8, clip: float = 0.8) -> Workload:
    """A tiny workload with the same structure, for CPU tests and brute-force checks."""
    assert T > n_text_head + n_text_tail
    seg = (("text", n_text_head), ("vision", T - n_text_head - n_text_tail), ("text", n_text_tail))
    return Workload(name, B, Hq, Hkv, T, G, seg, top_k, W=W, clip=clip)


def generate(w: Workload, seed: int = BASE_SEED, layer: int = 0, device: str = "cpu"):
    """Draw one layer's inputs.

    Returns a dict of tensors on `device`:
      k, v      [B,Hkv,T,D] fp16   post-RoPE Keys (un-rotated) and Values
      q_tail    [B,Hq,W,D]  fp16   the last W prompt queries (pivot scoring)
      q         [B,Hq,D]    fp16   one decode query per head
      is_text   [B,T]       uint8
      pivots    [B,4]       int64  planted pivot positions (position 0 + 3 vision positions)
      outlier_channels [Hkv,4] int64
    K ~ N(0,1) with 4 channels per KV head scaled by 20 (fixed over tokens and batch) and the 4 pivot rows
    scaled by 10; V, q, q_tail ~ N(0,1).
    """
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed) * 1000003 + 7919 * int(layer))
    cpu_g = torch.Generator(device="cpu")
    cpu_g.manual_seed(int(seed) * 1000003 + 7919 * int(layer) + 1)
    B = w.B
    mask = torch.from_numpy(is_text_mask(w))
    vision_pos = torch.nonzero(mask == 0).flatten()
    # structure is drawn on the CPU so that it is identical whatever device holds the big tensors
    outlier = torch.stack([torch.randperm(D, generator=cpu_g)[:N_OUTLIER_CHANNELS] for _ in range(w.Hkv)])
    piv = []
    for _ in range(B):
        sel = vision_pos[torch.randperm(vision_pos.numel(), generator=cpu_g)[:N_PIVOTS - 1]]
        piv.append(torch.cat([torch.zeros(1, dtype=torch.long), sel.sort().values]))
    pivots = torch.stack(piv)

    def randn(*shape):
        return torch.randn(*shape, generator=g, device=dev, dtype=torch.float32)

    k = torch.empty(B, w.Hkv, w.T, D, device=dev, dtype=torch.float16)
    v = torch.empty(B, w.Hkv, w.T, D, device=dev, dtype=torch.float16)
    gain = torch.ones(w.Hkv, D, device=dev)
    gain[torch.arange(w.Hkv).repeat_interleave(N_OUTLIER_CHANNELS), outlier.flatten()] = OUTLIER_GAIN
    for b in range(B):
        kb = randn(w.Hkv, w.T, D) * gain[:, None, :]
        kb[:, pivots[b].to(dev), :] *= PIVOT_GAIN
        k[b] = kb.to(torch.float16)
        v[b] = randn(w.Hkv, w.T, D).to(torch.float16)
    q_tail = randn(B, w.Hq, w.W, D).to(torch.float16)
    q = randn(B, w.Hq, D).to(torch.float16)
    is_text = mask.to(dev)[None, :].expand(B, w.T).contiguous()
    return {"k": k, "v": v, "q_tail": q_tail, "q": q, "is_text": is_text, "pivots": pivots,
            "outlier_channels": outlier}


def tiered_rows(is_text: np.ndarray, keep_plain=None):
    """Row plan of a cache with the 4-bit text tier: text tokens become (coarse, fine) row pairs starting on even rows
    (a padding row is inserted where needed), every other token (and every token listed in keep_plain[b]) one plain row.

    is_text [B, T] uint8.  Returns (row_src [B, n_rows] int32, row_tier [B, n_rows] uint8, row_of_token [B, T] int32);
    batch elements are padded with padding rows to a common, even n_rows.  Tiers: 0 plain 2-bit, 1 coarse, 2 fine, 3 pad.
    """
    B, T = is_text.shape
    plans = []
    for b in range(B):
        keep = set(int(x) for x in (keep_plain[b] if keep_plain is not None else ()))
        src, tier, row_of = [], [], np.zeros(T, dtype=np.int32)
        for t in range(T):
            if is_text[b, t] and t not in keep:
                if len(src) % 2:
                    src.append(t); tier.append(3)
                row_of[t] = len(src)
                src += [t, t]; tier += [1, 2]
            else:
                row_of[t] = len(src)
                src.append(t); tier.append(0)
        plans.append((src, tier, row_of))
    n_rows = max(len(p[0]) for p in plans)
    n_rows += n_rows % 2
    row_src = np.zeros((B, n_rows), dtype=np.int32)
    row_tier = np.full((B, n_rows), 3, dtype=np.uint8)
    row_of_token = np.zeros((B, T), dtype=np.int32)
    for b, (src, tier, row_of) in enumerate(plans):
        row_src[b, :len(src)] = src
        row_tier[b, :len(tier)] = tier
        row_of_token[b] = row_of
    return row_src, row_tier, row_of_token


def hidden_states(w: Workload, pivots, d_model: int = 4096, seed: int = BASE_SEED, layer: int = 0,
                  device: str = "cpu"):
    """A block's residual-stream output with massive activations planted at the pivot tokens: N(0,1) everywhere, two
    fixed channels of every pivot token raised to distinct magnitudes between 300 and 2500 (the pattern the paper's
    pivot identification relies on), and a sprinkling of merely large values (around 40) elsewhere.

    pivots [B, n] int64 (as returned by generate()).  Returns [B, T, d_model] fp16 on `device`."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed) * 1000003 + 7919 * int(layer) + 5)
    h = torch.randn(w.B, w.T, d_model, generator=g, device=dev, dtype=torch.float32)
    cpu_g = torch.Generator(device="cpu")
    cpu_g.manual_seed(int(seed) * 1000003 + 7919 * int(layer) + 6)
    ch = torch.randperm(d_model, generator=cpu_g)[:2]
    piv = torch.as_tensor(pivots).long()
    for b in range(w.B):
        for i, t in enumerate(piv[b].tolist()):
            h[b, t, ch[0]] = 300.0 + 173.0 * i + 37.0 * b
            h[b, t, ch[1]] = -(2500.0 - 211.0 * i - 29.0 * b)
    n_large = max(1, w.T // 50)
    pos = torch.randint(0, w.T, (w.B, n_large), generator=cpu_g)
    for b in range(w.B):
        h[b, pos[b], ch[0]] = 40.0
    return h.to(torch.float16)


def rope_tables(positions, theta: float = 10000.0):
    """cos / sin tables of a rotary position embedding as an fp16 model holds them: [..., 64] fp16 for integer positions
    [...], angle pos * theta^(-i/64), i < 64 (inputs of the fused RoPE entry points; both sides read the same bits)."""
    pos = np.asarray(positions, dtype=np.float64)
    inv_freq = theta ** (-np.arange(64, dtype=np.float64) / 64.0)
    ang = pos[..., None] * inv_freq
    return np.cos(ang).astype(np.float16), np.sin(ang).astype(np.float16)
