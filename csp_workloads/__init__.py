"""Seeded synthetic inputs for the CSP KV-cache pruning path.

This module only *draws inputs*: sequence layouts (which positions are visual,
which are text), Gaussian Q/K/V with the modality shift, the bf16 bit patterns
both sides read, budgets as integer fractions of the length.  It contains none
of the method's arithmetic (no softmax, no scoring, no selection), so the CPU
oracle and the HIP path can both take their inputs from here without sharing
anything else.

The paper evaluates on a multi-image benchmark with LLaVA weights
(Experiments, "Benchmark" and "Setup"); neither is available offline, so the
inputs below stand in for it: interleaved image/text spans as in the method
figure, 576 visual tokens per image (LLaVA-1.5), and a mean/scale gap between
visual and text keys that mimics the modality gap the paper's footnote in the
"Cross-self pruning" section describes (text keys attract larger weights than
visual keys).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

TEXT = 0
VISUAL = 1


# ----------------------------------------------------------------------------
# bf16 bit patterns (numpy has no bfloat16): round-to-nearest-even on the top
# 16 bits of an IEEE float32.  Inputs here are finite, so no NaN handling.
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


# ----------------------------------------------------------------------------
# Layouts
# ----------------------------------------------------------------------------
Span = Tuple[int, int]  # (modality, length)


def spans_to_modality(spans: Sequence[Span]) -> np.ndarray:
    parts = [np.full(n, m, dtype=np.uint8) for m, n in spans]
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.uint8)


def layout_tiny() -> List[Span]:
    """512 positions: text48 img144 text64 img144 text112."""
    return [(TEXT, 48), (VISUAL, 144), (TEXT, 64), (VISUAL, 144), (TEXT, 112)]


def layout_7b_4k() -> List[Span]:
    """4096 positions: 4 images of 576 visual tokens between 5 text spans
    (384, 384, 384, 384, 256 = 1792 text tokens)."""
    text = [384, 384, 384, 384, 256]
    spans: List[Span] = []
    for i, t in enumerate(text):
        spans.append((TEXT, t))
        if i < 4:
            spans.append((VISUAL, 576))
    return spans


def layout_random(rng: np.random.Generator, image_lens: Sequence[int], n_text: int,
                  last_text_min: int) -> List[Span]:
    """Images in the given order, separated by text spans obtained by cutting
    `n_text` text tokens at random into len(image_lens)+1 pieces; the last
    piece has at least `last_text_min` tokens so the observation window is
    all text."""
    n_img = len(image_lens)
    assert n_text >= last_text_min
    free = n_text - last_text_min
    cuts = np.sort(rng.integers(0, free + 1, size=n_img))
    edges = np.concatenate([[0], cuts, [free]])
    pieces = np.diff(edges).astype(np.int64)
    pieces[-1] += last_text_min
    spans: List[Span] = []
    for i in range(n_img):
        if pieces[i] > 0:
            spans.append((TEXT, int(pieces[i])))
        spans.append((VISUAL, int(image_lens[i])))
    spans.append((TEXT, int(pieces[-1])))
    return spans


def layout_mixed_window(rng: np.random.Generator, image_lens: Sequence[int], n_text: int,
                        window_text: int) -> List[Span]:
    """As layout_random, but the sequence ends with the last image followed by only
    `window_text` text tokens: an observation window longer than that holds queries
    of both modalities."""
    assert 0 < window_text <= n_text and len(image_lens) >= 1
    spans = [s for s in layout_random(rng, image_lens[:-1], n_text - window_text, 0) if s[1] > 0]
    return spans + [(VISUAL, int(image_lens[-1])), (TEXT, int(window_text))]


# ----------------------------------------------------------------------------
# Cases
# ----------------------------------------------------------------------------
@dataclass
class Case:
    """One batch of synthetic input for one layer.

    Arrays are numpy; for dtype "bf16" the Q/K/V arrays hold uint16 bit
    patterns, for "f32" float32 values.  Layout (head-major, token-packed):
      q_win  [B, H_q, O, D]          queries of the last O positions
      k, v   [H_kv, total_tokens, D] rows of sequence b are cu_seqlens[b]..cu_seqlens[b+1]
      modality uint8[total_tokens]   1 = visual
      dec_q  [steps, B, H_q, D]      decode queries
      dec_k, dec_v [steps, B, H_kv, D]  the key/value each decode step appends
    """
    name: str
    dtype: str
    B: int
    H_q: int
    H_kv: int
    D: int
    O: int
    R: int
    sel_group: int
    cross_ratio: float
    n_score: float
    n_decode: float
    cu_seqlens: np.ndarray
    budget_T: np.ndarray
    modality: np.ndarray
    q_win: np.ndarray
    k: np.ndarray
    v: np.ndarray
    dec_q: np.ndarray
    dec_k: np.ndarray
    dec_v: np.ndarray
    spans: List[List[Span]] = field(default_factory=list)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    def seqlen(self, b: int) -> int:
        return int(self.cu_seqlens[b + 1] - self.cu_seqlens[b])

    def as_f32(self, a: np.ndarray) -> np.ndarray:
        return bf16_bits_to_f32(a) if self.dtype == "bf16" else a.astype(np.float32)


def _draw(rng: np.random.Generator, shape, dtype: str) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def _shift_visual_keys(k: np.ndarray, modality: np.ndarray, dtype: str,
                       heavy: Optional[np.ndarray] = None) -> np.ndarray:
    """Visual keys: k <- 0.7*k + 0.5 (then x4 on the `heavy` positions), applied
    in float32 and rounded once to the storage dtype."""
    kf = bf16_bits_to_f32(k) if dtype == "bf16" else k.astype(np.float32)
    vis = modality.astype(bool)
    kf = kf.copy()
    kf[:, vis, :] = np.float32(0.7) * kf[:, vis, :] + np.float32(0.5)
    if heavy is not None and heavy.any():
        kf[:, heavy, :] = np.float32(4.0) * kf[:, heavy, :]
    return f32_to_bf16_bits(kf) if dtype == "bf16" else kf


def make_case(name: str, *, dtype: str, H_q: int, H_kv: int, D: int, O: int, R: int,
              layouts: Sequence[Sequence[Span]], budgets: Sequence[int], seed: int,
              sel_group: int = 1, cross_ratio: float = 0.5, n_score: float = 0.0,
              n_decode: float = 1.0, decode_steps: int = 0,
              heavy_visual_frac: float = 0.0) -> Case:
    rng = np.random.default_rng(seed)
    B = len(layouts)
    mods = [spans_to_modality(s) for s in layouts]
    lens = np.array([len(m) for m in mods], dtype=np.int64)
    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    modality = np.concatenate(mods) if B else np.zeros(0, np.uint8)
    total = int(cu[-1])
    q_win = _draw(rng, (B, H_q, O, D), dtype)
    k = _draw(rng, (H_kv, total, D), dtype)
    v = _draw(rng, (H_kv, total, D), dtype)
    heavy = None
    if heavy_visual_frac > 0:
        heavy = (rng.random(total) < heavy_visual_frac) & modality.astype(bool)
    k = _shift_visual_keys(k, modality, dtype, heavy)
    dec_q = _draw(rng, (decode_steps, B, H_q, D), dtype)
    dec_k = _draw(rng, (decode_steps, B, H_kv, D), dtype)
    dec_v = _draw(rng, (decode_steps, B, H_kv, D), dtype)
    return Case(name=name, dtype=dtype, B=B, H_q=H_q, H_kv=H_kv, D=D, O=O, R=R,
                sel_group=sel_group, cross_ratio=cross_ratio, n_score=n_score,
                n_decode=n_decode, cu_seqlens=cu,
                budget_T=np.asarray(budgets, dtype=np.int32), modality=modality,
                q_win=q_win, k=k, v=v, dec_q=dec_q, dec_k=dec_k, dec_v=dec_v,
                spans=[list(s) for s in layouts])


# --- the benchmark configurations ----------------------------------------------
def case_tiny(seed: int = 0) -> Case:
    """Tiny CPU-checkable case: B=1, 8 heads (MHA), D=64, fp32, L=512, O=R=32,
    T=256."""
    return make_case("tiny", dtype="f32", H_q=8, H_kv=8, D=64, O=32, R=32,
                     layouts=[layout_tiny()], budgets=[256], seed=seed, decode_steps=4)


def case_7b_4k(seed: int = 0, decode_steps: int = 16) -> Case:
    """7B-shape single layer: B=1, 32 heads, D=128, bf16, L=4096, O=R=64,
    T=2048, 16 decode steps."""
    return make_case("7b_4k", dtype="bf16", H_q=32, H_kv=32, D=128, O=64, R=64,
                     layouts=[layout_7b_4k()], budgets=[2048], seed=seed,
                     decode_steps=decode_steps)


def layout_7b_16k(rng: np.random.Generator) -> List[Span]:
    """16384 positions: 20 images x 576 visual tokens + 4864 text tokens cut at
    random into 21 spans, the last at least 64 long."""
    return layout_random(rng, [576] * 20, 4864, 64)


def layout_gqa_ragged(rng: np.random.Generator, max_len: int = 8192) -> List[Span]:
    """2-12 images of 256-1024 visual tokens and 512-2048 text tokens, redrawn
    until the sequence fits max_len."""
    while True:
        n_img = int(rng.integers(2, 13))
        img = rng.integers(256, 1025, size=n_img).tolist()
        n_text = int(rng.integers(512, 2049))
        if sum(img) + n_text <= max_len:
            return layout_random(rng, img, n_text, 64)


def layout_64k(rng: np.random.Generator) -> List[Span]:
    """65536 positions: 100 images x 576 + 7936 text, last text span >= 128."""
    return layout_random(rng, [576] * 100, 7936, 128)


def case_gqa_ragged(seed: int = 0, B: int = 8, decode_steps: int = 2,
                    max_len: int = 8192) -> Case:
    rng = np.random.default_rng(seed + 1000)
    layouts = [layout_gqa_ragged(rng, max_len) for _ in range(B)]
    budgets = [sum(n for _, n in s) // 2 for s in layouts]
    return make_case("gqa_ragged", dtype="bf16", H_q=28, H_kv=4, D=128, O=64, R=64,
                     layouts=layouts, budgets=budgets, seed=seed, sel_group=7,
                     decode_steps=decode_steps)


# ----------------------------------------------------------------------------
# Device-side generation for the full-size configurations (tens of GiB): same
# recipe, drawn with torch's seeded generator on the GPU.  The oracle reads the
# rows it checks after they are copied back, so both sides still see identical
# bit patterns.
# ----------------------------------------------------------------------------
def device_qkv(layouts: Sequence[Sequence[Span]], *, H_q: int, H_kv: int, D: int, O: int,
               seed: int, device, heavy_visual_frac: float = 0.0):
    """Returns (q_win[B,H_q,O,D], k[H_kv,total,D], v[H_kv,total,D], modality uint8[total],
    cu_seqlens int32[B+1]) as bf16 torch tensors on `device`."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(seed)
    B = len(layouts)
    mods = [spans_to_modality(s) for s in layouts]
    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum([len(m) for m in mods])
    total = int(cu[-1])
    modality = torch.from_numpy(np.concatenate(mods)).to(device)
    q = torch.randn((B, H_q, O, D), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    k = torch.empty((H_kv, total, D), device=device, dtype=torch.bfloat16)
    v = torch.empty((H_kv, total, D), device=device, dtype=torch.bfloat16)
    vis = modality.bool()
    heavy = None
    if heavy_visual_frac > 0:
        heavy = (torch.rand(total, generator=g, device=device) < heavy_visual_frac) & vis
    for h in range(H_kv):  # per head keeps the fp32 temporaries small
        kf = torch.randn((total, D), generator=g, device=device, dtype=torch.float32)
        kf[vis] = 0.7 * kf[vis] + 0.5
        if heavy is not None:
            kf[heavy] = 4.0 * kf[heavy]
        k[h] = kf.to(torch.bfloat16)
        v[h] = torch.randn((total, D), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    return q, k, v, modality, torch.from_numpy(cu).to(device), cu
