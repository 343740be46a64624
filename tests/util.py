"""Shared helpers for the tests: bf16 bit handling, tiny random cases, and a
pure-Python brute force of the definitions used to pin the oracle."""
from __future__ import annotations

import math
from typing import List, Optional

import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit pattern (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def as_f64(a: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


class TinyCase:
    """Random small problem: K,V [B,Hkv,S,d], q [B,Hq,d], one visual span per sequence."""

    def __init__(self, seed, B, Hq, Hkv, d, n_vis, pre, post, dtype="f32", spread=1.0):
        rng = np.random.default_rng(seed)
        self.B, self.Hq, self.Hkv, self.d, self.dtype = B, Hq, Hkv, d, dtype
        n_vis = [n_vis] * B if np.isscalar(n_vis) else list(n_vis)
        pre = [pre] * B if np.isscalar(pre) else list(pre)
        post = [post] * B if np.isscalar(post) else list(post)
        self.vis_len = np.array(n_vis, np.int32)
        self.vis_start = np.array(pre, np.int32)
        self.seq_len = np.array([pre[b] + n_vis[b] + post[b] for b in range(B)], np.int32)
        S = int(self.seq_len.max())
        self.S = S
        self.k = store(rng.normal(size=(B, Hkv, S, d)) * spread, dtype)
        self.v = store(rng.normal(size=(B, Hkv, S, d)), dtype)
        self.q = store(rng.normal(size=(B, Hq, d)) * spread, dtype)
        self.scale = float(np.float32(1.0 / math.sqrt(d)))   # exactly representable in fp32


# ---------------------------------------------------------------------------
# Pure-Python brute force (loops, math.fsum): the definitions written a second
# time, independently of oracle/, for tiny inputs only.
# ---------------------------------------------------------------------------

def brute_logits(case: TinyCase, b: int, h: int) -> List[float]:
    K, Q = as_f64(case.k), as_f64(case.q)
    G = case.Hq // case.Hkv
    S = int(case.seq_len[b])
    return [case.scale * math.fsum(Q[b, h, c] * K[b, h // G, j, c] for c in range(case.d))
            for j in range(S)]


def brute_scores(case: TinyCase, b: int) -> List[float]:
    S = int(case.seq_len[b]); N = int(case.vis_len[b]); v0 = int(case.vis_start[b])
    acc = [0.0] * N
    for h in range(case.Hq):
        lg = brute_logits(case, b, h)
        m = max(lg)
        e = [math.exp(x - m) for x in lg]
        z = math.fsum(e)
        for i in range(N):
            acc[i] += e[v0 + i] / z
    return [a / case.Hq for a in acc]


def brute_topk(scores, k: int) -> List[int]:
    order = sorted(range(len(scores)), key=lambda i: (-scores[i], i))
    return sorted(order[:k])


def brute_attn(case: TinyCase, b: int, h: int, sel: Optional[List[int]]) -> List[float]:
    """sel None -> all tokens; else text tokens plus vis_start+sel."""
    V = as_f64(case.v)
    G = case.Hq // case.Hkv
    S = int(case.seq_len[b]); N = int(case.vis_len[b]); v0 = int(case.vis_start[b])
    if sel is None:
        J = list(range(S))
    else:
        J = [j for j in range(S) if j < v0 or j >= v0 + N] + [v0 + i for i in sel]
    lg = brute_logits(case, b, h)
    if not J:
        return [0.0] * case.d
    m = max(lg[j] for j in J)
    e = {j: math.exp(lg[j] - m) for j in J}
    z = math.fsum(e.values())
    return [math.fsum(e[j] / z * V[b, h // G, j, c] for j in J) for c in range(case.d)]
