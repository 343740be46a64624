"""Oracle of the per-step layer schedule (Algorithm 1, App. A) -- TEST INFRASTRUCTURE ONLY.

Given the frozen focal layer set C, the warm-up length w and whether a focal
token set survives from the previous step, say for every layer of decode step t
what kind of attention it runs and whose focal token set it attends over.
Written from the algorithm's three blocks in their order.  ``select_focal_layers``
is the Focal Layer Selection block (Sec. 3.1.1): rank layers by their mean
image-attention ratio over the warm-up steps, then take them greedily while the
budget floor(rho L) lasts and the focal gap to every layer already taken holds.
"""
from __future__ import annotations

from typing import List, NamedTuple, Optional, Sequence


class LayerAction(NamedTuple):
    layer: int
    mode: str                 # "full" | "full+select" | "pruned"
    set_from: Optional[object]  # "F_last", a layer index, or None (full attention)


class StepPlan(NamedTuple):
    actions: List[LayerAction]
    save_from: Optional[int]  # layer whose focal token set becomes F_last; None = unchanged


def plan_step(t: int, n_layers: int, focal_layers: Sequence[int], warmup: int,
              have_f_last: bool) -> StepPlan:
    """Schedule of decode step t (1-based, as in the paper)."""
    C = set(int(c) for c in focal_layers)
    if not C:
        raise ValueError("the focal layer set must not be empty")
    if min(C) < 0 or max(C) >= n_layers:
        raise ValueError("focal layer outside [0, L)")

    # Focal Layer Selection phase: no pruning at all during the first w steps.
    if t <= warmup:
        return StepPlan([LayerAction(i, "full", None) for i in range(n_layers)], None)

    actions: List[LayerAction] = []
    # Cross-Step Fixation Reuse block: where does layer 0's focal token set come from?
    if 0 not in C and have_f_last:
        actions.append(LayerAction(0, "pruned", "F_last"))
        current = "F_last"
    else:
        # fallback (or layer 0 is focal): top-k of layer 0's own image attention
        actions.append(LayerAction(0, "full+select", None))
        current = 0
    # Cross-Layer Propagation block.
    for i in range(1, n_layers):
        if i in C:
            actions.append(LayerAction(i, "full+select", None))
            current = i
        else:
            actions.append(LayerAction(i, "pruned", current))
    return StepPlan(actions, max(C))


def select_focal_layers(ratios, rho: float, gap: int) -> List[int]:
    """ratios[t][i]: image-attention ratio r_i^(t) of layer i at warm-up step t (Eq. 1), or
    ratios[t][i][b] per sequence of a batch (then also averaged over the batch: one focal set
    serves the whole batch).  Returns the focal layer set C, ascending."""
    import numpy as np
    r = np.asarray(ratios, dtype=np.float64)
    if r.ndim == 3:
        r = r.mean(axis=2)
    if r.ndim != 2 or r.shape[0] < 1:
        raise ValueError("ratios must be [steps][layers] or [steps][layers][batch]")
    n_layers = r.shape[1]
    mean = r.mean(axis=0)
    # descending by mean ratio; equal means keep the lower layer first
    ranked = sorted(range(n_layers), key=lambda i: (-mean[i], i))
    budget = int(np.floor(rho * n_layers + 1e-9))
    chosen: List[int] = []
    for i in ranked:
        if len(chosen) < budget and all(abs(i - j) > gap for j in chosen):
            chosen.append(i)
    return sorted(chosen)
