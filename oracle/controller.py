"""Oracle of the per-step layer schedule (Algorithm 1, App. A) -- TEST INFRASTRUCTURE ONLY.

Given the frozen focal layer set C, the warm-up length w and whether a focal
token set survives from the previous step, say for every layer of decode step t
what kind of attention it runs and whose focal token set it attends over.
Written from the algorithm's three blocks in their order; no arithmetic here.
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
