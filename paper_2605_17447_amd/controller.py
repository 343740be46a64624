"""Host-side step controller: which call each layer of a decode step enqueues.

Implements the per-step control flow of Algorithm 1 (App. A) for a frozen focal layer set C:
warm-up steps run full attention everywhere; afterwards a focal layer attends the full cache
and refreshes the kept image tokens (Cross-Layer Propagation, Sec. 3.1.2), every other layer
attends text + the kept tokens, and the set left by the deepest focal layer serves layer 0 of
the next step (Cross-Step Fixation Reuse, Sec. 3.2).  When no focal layer set is given, the
warm-up steps also record every layer's image-attention ratio (Eq. 1: the image mass that
focal scoring returns) and the set is chosen after the last of them (Focal Layer Selection,
Sec. 3.1.1) by the library's host routine.  A layer that needs both its full-cache output and
the image scores gets them from one call (one pass over K and V).  No arithmetic happens here:
the controller only owns device buffers and orders the C-ABI calls on one stream.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import torch

from . import binding as _b


class FixationController:
    def __init__(self, caches: Sequence[_b.KvCache], n_q_heads: int, scale: float,
                 focal_layers: Optional[Sequence[int]], tau: float, warmup: int, max_seq_len: int,
                 max_vis_len: int, batch_size: int, device, focal_gap: int = 1, ops=None,
                 focal_ratio: float = 0.1):
        self.caches = list(caches)
        self.n_layers = len(self.caches)
        self.focal_gap, self.focal_ratio = int(focal_gap), float(focal_ratio)
        if focal_layers is None:
            # chosen from the warm-up steps' image-attention ratios
            if warmup < 1:
                raise ValueError("focal layer selection needs at least one warm-up step")
            if int(self.focal_ratio * self.n_layers + 1e-9) < 1:
                raise ValueError("focal_ratio * layers must allow at least one focal layer")
            self.focal = None
            self.ratios = torch.zeros((warmup, self.n_layers, batch_size), dtype=torch.float32, device=device)
        else:
            self.focal = sorted(set(int(c) for c in focal_layers))
            if not self.focal:
                raise ValueError("the focal layer set must not be empty")
            if self.focal[0] < 0 or self.focal[-1] >= self.n_layers:
                raise ValueError("focal layer outside the stack")
            # the focal gap is a spacing in layers between focal layers (Sec. 3.1.1)
            for a, c in zip(self.focal, self.focal[1:]):
                if c - a <= focal_gap:
                    raise ValueError(f"focal layers {a} and {c} are closer than the focal gap {focal_gap}")
        if not (0.0 <= tau <= 1.0):
            raise ValueError("tau must lie in [0, 1]")
        self.tau, self.warmup, self.scale, self.n_q_heads = float(tau), int(warmup), float(scale), n_q_heads
        self.ops = ops if ops is not None else _b
        self.device = device
        self.kmax = max(1, self.ops.keep_count(max_vis_len, tau))
        self.scores = torch.zeros((batch_size, max(max_vis_len, 1)), dtype=torch.float32, device=device)
        self.kept_idx = torch.zeros((batch_size, self.kmax), dtype=torch.int32, device=device)
        self.kept_cnt = torch.zeros((batch_size,), dtype=torch.int32, device=device)
        self.kept_from: Optional[object] = None     # None: no set yet; "F_last"; or a layer index
        self._ws = None
        self._ws_bytes = 0
        # workspace sizes are asked for once per layer, for the longest sequences the run will see
        # (a size never shrinks as sequences grow), not at every step
        self._bound_seq, self._bound_vis = int(max_seq_len), int(max_vis_len)
        self._need = {}
        # set while a step is being captured into a HIP graph: the library is then told that its launches
        # will follow each other closely (fastocr_set_tuning("graph_replay", 1)) for the calls of that step
        self.graph_replay = False

    def _workspace(self, cache, batch):
        if batch.max_seq_len > self._bound_seq or batch.max_vis_len > self._bound_vis:
            self._bound_seq = max(self._bound_seq, int(batch.max_seq_len))
            self._bound_vis = max(self._bound_vis, int(batch.max_vis_len))
            self._need.clear()
        need = self._need.get(id(cache))
        if need is None:
            bound = _b.SeqBatch(batch.seq_len, batch.vis_start, batch.vis_len, self._bound_seq, self._bound_vis)
            need = 0
            for op in (_b.OP_FOCAL_ATTN_SCORE, _b.OP_FOCAL_ATTN_SCORE_TOPK, _b.OP_TOPK_FIXATION, _b.OP_SPARSE_DECODE_ATTN, _b.OP_DENSE_DECODE_ATTN):
                need = max(need, self.ops.workspace_bytes(op, cache, bound, self.n_q_heads, self.kmax))
            self._need[id(cache)] = need
        if self._ws is None or self._ws_bytes < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
            self._ws_bytes = need
        return self._ws

    def step(self, t: int, batch: "_b.SeqBatch", queries: Sequence[torch.Tensor],
             outs: Sequence[torch.Tensor], stream=None, on_select=None) -> List[Tuple[int, str, Optional[object]]]:
        """Enqueue decode step t (1-based).  queries[l], outs[l]: [B, Hq, d] per layer.
        Returns the schedule it ran as (layer, mode, kept-set source) triples.
        ``on_select(layer, scores, kept_idx, kept_cnt)`` is called right after a selecting layer
        has been enqueued (the tensors are the controller's own buffers, valid in stream order)."""
        if not self.graph_replay:
            return self._step(t, batch, queries, outs, stream, on_select)
        self.ops.set_tuning("graph_replay", 1)
        try:
            return self._step(t, batch, queries, outs, stream, on_select)
        finally:
            self.ops.set_tuning("graph_replay", 0)

    def _step(self, t, batch, queries, outs, stream, on_select):
        ops, trace = self.ops, []
        post_warmup = t > self.warmup
        if post_warmup and self.focal is None:
            raise RuntimeError("the focal layer set is chosen at the last warm-up step: run steps 1..warmup first")
        if post_warmup and self.kept_from is not None:
            self.kept_from = "F_last"             # what the previous step left behind
        for l, cache in enumerate(self.caches):
            ws = self._workspace(cache, batch)
            q, out = queries[l], outs[l]
            if not post_warmup:
                if self.focal is None:
                    # full attention plus r_l^(t) of Eq. 1 for every sequence from the same pass over the
                    # cache; the ratios stay on the device until the last warm-up step
                    ops.focal_attn_score(cache, batch, q, self.scale, out, self.scores, ws,
                                         img_mass=self.ratios[t - 1, l], stream=stream)
                else:
                    ops.dense_decode_attn(cache, batch, q, self.scale, out, ws, stream=stream)
                trace.append((l, "full", None))
                continue
            selects = (l in self.focal) or (l == 0 and self.kept_from is None)
            if selects:
                # the layer's own output over the full cache, the scores its successors are pruned by and
                # their top-k, from one call (its last launch merges the output's partials and selects)
                warm = self.kept_from is not None
                ops.focal_attn_score_topk(cache, batch, q, self.scale, self.tau, out, self.scores, self.kept_idx,
                                          self.kept_cnt, ws, prev_idx=self.kept_idx if warm else None,
                                          prev_cnt=self.kept_cnt if warm else None, stream=stream)
                self.kept_from = l
                if on_select is not None:
                    on_select(l, self.scores, self.kept_idx, self.kept_cnt)
                trace.append((l, "full+select", None))
            else:
                ops.sparse_decode_attn(cache, batch, q, self.scale, self.kept_idx, self.kept_cnt, out, ws,
                                       stream=stream)
                trace.append((l, "pruned", self.kept_from))
        if self.focal is None and t == self.warmup:
            # Focal Layer Selection: one read-back of warmup x layers x batch ratios, ranked on the host
            self.focal = ops.select_focal_layers(self.ratios.cpu().numpy(), self.focal_ratio, self.focal_gap)
        # after the last layer the kept set is the deepest focal layer's: it is next step's F_last
        return trace
