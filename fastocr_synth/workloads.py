"""Workload shapes, cache construction and the drifting-fixation query process.

Sequence layout (token positions of one sequence):

    [ floor(P/2) text ][ N visual, row-major W x H grid ][ P - floor(P/2) text ][ generated ... ]

so text sits on both sides of the visual span.  At decode step t (1-based) the
sequence holds N + P + t tokens; the last one is the current token.  The cache is
generated up to its final length once, so "appending" a token is only a longer
``seq_len``.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from .rng import normal_rows, uniform_u64

BASE_SEED = 20260517

TAG_K, TAG_V, TAG_QNOISE, TAG_CENTRE, TAG_SHAPE, TAG_PAGES = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                      # "f32" | "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_visual: Tuple[int, int]       # inclusive range the per-sequence N' is drawn from
    grid_w: Tuple[int, int]         # clip range of the grid width
    text_prefix: Tuple[int, int]    # inclusive range of the text prefix length P
    steps: int
    taus: Tuple[float, ...]
    warmup: int = 0
    window_r: int = 2
    sigma: float = 0.1
    beta: float = 1.0               # gain on the window mean (1 = as specified)
    n_layers: int = 1
    focal_layers: Tuple[int, ...] = (0,)
    focal_gap: int = 1
    line_jump: int = 0              # jump to the next row start every this many steps (0 = never)
    centre_anywhere: bool = False   # first centre uniform over the grid instead of row 0
    paged: bool = False
    page_tokens: int = 64
    config_id: int = 0

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


def config(i: int, **overrides) -> Workload:
    """The five benchmark configurations; ``overrides`` make scaled-down variants."""
    if i == 1:
        wl = Workload("tiny-fp32", "f32", 1, 4, 1, 64, (256, 256), (16, 16), (31, 31), 1, (0.05,),
                      window_r=1, centre_anywhere=True, config_id=1)
    elif i == 2:
        wl = Workload("qwen7b-layer-b1", "bf16", 1, 28, 4, 128, (4096, 4096), (64, 64), (64, 64), 512,
                      (0.05,), warmup=4, config_id=2)
    elif i == 3:
        wl = Workload("qwen7b-stack-b8", "bf16", 8, 28, 4, 128, (4096, 4096), (64, 64), (128, 128), 256,
                      (0.05, 0.10), warmup=4, n_layers=28, focal_layers=(2, 14), focal_gap=8,
                      config_id=3)
    elif i == 4:
        wl = Workload("dense-doc-72b-layer-b16", "bf16", 16, 64, 8, 128, (16384, 16384), (128, 128),
                      (256, 256), 1024, (0.02, 0.05, 1.0), warmup=0, line_jump=128, config_id=4)
    elif i == 5:
        wl = Workload("ragged-serving-b32", "bf16", 32, 28, 4, 128, (2048, 16384), (64, 128), (32, 512),
                      512, (0.05,), warmup=4, n_layers=28, focal_layers=(2, 14), focal_gap=8,
                      paged=True, page_tokens=64, config_id=5)
    else:
        raise ValueError(f"no config {i}")
    return dataclasses.replace(wl, **overrides) if overrides else wl


@dataclass
class Batch:
    """One layer's cache for a batch of sequences plus the sequences' geometry."""
    wl: Workload
    seed: int
    layer: int
    device: torch.device
    n_vis: List[int]
    grid_w: List[int]
    grid_h: List[int]
    prefix: List[int]
    vis_start: List[int]
    cap: int                                  # token capacity per sequence (max over the batch)
    k: torch.Tensor = None                    # [B,Hkv,cap,d]  or  paged [n_pages,Hkv,page_tokens,d]
    v: torch.Tensor = None
    block_table: Optional[torch.Tensor] = None  # [B, max_pages] int32 (paged only)

    def seq_len(self, t: int) -> List[int]:
        """Tokens held at decode step t (1-based), current token included."""
        return [self.n_vis[b] + self.prefix[b] + t for b in range(self.wl.batch)]

    def rows(self, which: str, b: int, tokens: torch.Tensor) -> torch.Tensor:
        """Stored rows [Hkv, len(tokens), d] of sequence b (either layout)."""
        src = self.k if which == "k" else self.v
        tokens = tokens.to(self.device, torch.int64)
        if self.block_table is None:
            return src[b].index_select(1, tokens)
        pt = self.wl.page_tokens
        pages = self.block_table[b].to(torch.int64)[tokens // pt]
        return src[pages, :, tokens % pt, :].permute(1, 0, 2)


def _geometry(wl: Workload, seed: int):
    n_vis, gw, gh, prefix = [], [], [], []
    for b in range(wl.batch):
        lo, hi = wl.n_visual
        n0 = lo + uniform_u64(seed + b, TAG_SHAPE, 0) % (hi - lo + 1)
        w = min(max(int(round(math.sqrt(n0))), wl.grid_w[0]), wl.grid_w[1])
        h = -(-n0 // w)
        while w * h > hi:
            h -= 1
        plo, phi = wl.text_prefix
        p = plo + uniform_u64(seed + b, TAG_SHAPE, 1) % (phi - plo + 1)
        n_vis.append(w * h); gw.append(w); gh.append(h); prefix.append(int(p))
    return n_vis, gw, gh, prefix


def _row_ids(layer: int, n_kv_heads: int, tokens: torch.Tensor) -> torch.Tensor:
    heads = torch.arange(n_kv_heads, device=tokens.device, dtype=torch.int64)
    return ((layer * 64 + heads) << 32).unsqueeze(1) + tokens.unsqueeze(0)   # [Hkv, T]


def make_batch(wl: Workload, seed: int = BASE_SEED, device="cpu", layer: int = 0,
               chunk_tokens: int = 8192, plain_fill: bool = False) -> Batch:
    """Generate one layer's K and V (N(0,1), rounded to the storage dtype).

    plain_fill: the same geometry, page tables and distribution, but the values come from one
    random-normal launch per tensor (torch's generator) instead of the counter-based generator's
    many small ones; they are NOT reproducible across devices and never go to the oracle.
    """
    device = torch.device(device)
    seed = seed + 1000003 * wl.config_id
    n_vis, gw, gh, prefix = _geometry(wl, seed)
    caps = [n_vis[b] + prefix[b] + wl.steps for b in range(wl.batch)]
    cap = max(caps)
    bt = Batch(wl, seed, layer, device, n_vis, gw, gh, prefix, [p // 2 for p in prefix], cap)
    dt = wl.torch_dtype
    H, d = wl.n_kv_heads, wl.head_dim
    if wl.paged:
        pt = wl.page_tokens
        pages_per = [-(-c // pt) for c in caps]
        total = sum(pages_per)
        # interleave the sequences' pages in one pool with a seeded permutation
        order = sorted(range(total), key=lambda s: uniform_u64(seed, TAG_PAGES, s))
        table = torch.zeros((wl.batch, max(pages_per)), dtype=torch.int32)
        pos = 0
        for b in range(wl.batch):
            table[b, : pages_per[b]] = torch.tensor(order[pos: pos + pages_per[b]], dtype=torch.int32)
            pos += pages_per[b]
        bt.block_table = table.to(device)
        bt.k = torch.zeros((total, H, pt, d), dtype=dt, device=device)
        bt.v = torch.zeros((total, H, pt, d), dtype=dt, device=device)
    else:
        bt.k = torch.zeros((wl.batch, H, cap, d), dtype=dt, device=device)
        bt.v = torch.zeros((wl.batch, H, cap, d), dtype=dt, device=device)
    if plain_fill:
        g = torch.Generator(device=device).manual_seed(seed + 7919 * layer)
        bt.k = torch.randn(bt.k.shape, generator=g, device=device, dtype=torch.float32).to(dt)
        bt.v = torch.randn(bt.v.shape, generator=g, device=device, dtype=torch.float32).to(dt)
        return bt
    for b in range(wl.batch):
        for t0 in range(0, caps[b], chunk_tokens):
            toks = torch.arange(t0, min(t0 + chunk_tokens, caps[b]), device=device, dtype=torch.int64)
            ids = _row_ids(layer, H, toks)
            for tag, dst in ((TAG_K, bt.k), (TAG_V, bt.v)):
                vals = normal_rows(seed + b, tag, ids, d).to(dt)          # [H, T, d]
                if wl.paged:
                    pt = wl.page_tokens
                    pages = bt.block_table[b].to(torch.int64)[toks // pt]
                    dst[pages, :, toks % pt, :] = vals.permute(1, 0, 2)
                else:
                    dst[b, :, t0: t0 + toks.numel(), :] = vals
    return bt


def centres(bt: Batch, n_steps: Optional[int] = None) -> List[List[int]]:
    """Fixation centre (visual cell index) of every sequence at steps 1..n_steps."""
    wl = bt.wl
    n_steps = wl.steps if n_steps is None else n_steps
    out = []
    for b in range(wl.batch):
        W, N = bt.grid_w[b], bt.n_vis[b]
        span = N if wl.centre_anywhere else W
        c = int(uniform_u64(bt.seed + b, TAG_CENTRE, 0) % span)
        seq = [c]
        for t in range(1, n_steps):
            c = (c + 1 + int(uniform_u64(bt.seed + b, TAG_CENTRE, t) % 2)) % N
            if wl.line_jump and t % wl.line_jump == 0:
                c = (((c // W) + 1) % bt.grid_h[b]) * W
            seq.append(c)
        out.append(seq)
    return out


def window_cells(c: int, W: int, H: int, r: int) -> List[int]:
    """Cells of the (2r+1)^2 window around cell c, clipped to the grid (no wrap)."""
    row, col = divmod(c, W)
    return [rr * W + cc
            for rr in range(max(0, row - r), min(H, row + r + 1))
            for cc in range(max(0, col - r), min(W, col + r + 1))]


def queries_for_step(bt: Batch, t: int, centre_t: Sequence[int]) -> torch.Tensor:
    """Queries [B, Hq, d] of decode step t (1-based): for query head h, the mean of
    the stored keys of KV head h // (Hq/Hkv) over the window around this step's
    centre, times beta, plus sigma * N(0, I); rounded to the storage dtype."""
    wl = bt.wl
    G = wl.n_q_heads // wl.n_kv_heads
    q = torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float64, device=bt.device)
    heads = torch.arange(wl.n_q_heads, device=bt.device, dtype=torch.int64)
    for b in range(wl.batch):
        cells = window_cells(int(centre_t[b]), bt.grid_w[b], bt.grid_h[b], wl.window_r)
        toks = torch.tensor(cells, dtype=torch.int64, device=bt.device) + bt.vis_start[b]
        mean = bt.rows("k", b, toks).to(torch.float64).mean(dim=1)          # [Hkv, d]
        ids = ((bt.layer * 4096 + heads) << 32) + t
        noise = normal_rows(bt.seed + b, TAG_QNOISE, ids, wl.head_dim)      # [Hq, d]
        q[b] = wl.beta * mean.repeat_interleave(G, dim=0) + wl.sigma * noise
    return q.to(wl.torch_dtype)


def to_oracle_array(t: torch.Tensor) -> np.ndarray:
    """Host copy with the same bits: float32 stays float32, bf16 becomes uint16."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()
