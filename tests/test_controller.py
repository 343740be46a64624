"""The step controller against the oracle of Algorithm 1's control flow (CPU only: the four
C-ABI calls are replaced by a recorder, so only the schedule is under test)."""
import pytest
import torch

from oracle.controller import plan_step
from paper_2605_17447_amd.binding import SeqBatch
from paper_2605_17447_amd.controller import FixationController

# geometry of one sequence; the recorder never looks inside, the controller reads its maxima
_BATCH = SeqBatch.from_lists([300], [10], [256], "cpu")


class Recorder:
    """Stands in for the binding: records calls, computes nothing."""

    def __init__(self):
        self.calls = []

    def keep_count(self, n, tau):
        return max(1, int(n * tau))

    def workspace_bytes(self, *a, **k):
        return 256

    def dense_decode_attn(self, cache, batch, q, scale, out, ws, **kw):
        self.calls.append(("dense", cache))

    def focal_attn_score(self, cache, batch, q, scale, out, scores, ws, **kw):
        self.calls.append(("dense+score", cache))

    def topk_fixation(self, scores, batch, tau, sel_idx, sel_cnt, ws, prev_idx=None, prev_cnt=None, **kw):
        self.calls.append(("topk", prev_idx is not None))

    def focal_attn_score_topk(self, cache, batch, q, scale, tau, out, scores, sel_idx, sel_cnt, ws, prev_idx=None,
                              prev_cnt=None, **kw):
        # a selecting layer is one call: its own full attention, its scores and their top-k
        self.calls.append(("dense+score", cache))
        self.calls.append(("topk", prev_idx is not None))

    def sparse_decode_attn(self, cache, batch, q, scale, sel_idx, sel_cnt, out, ws, **kw):
        self.calls.append(("sparse", cache))


def _run(n_layers, focal, warmup, steps):
    rec = Recorder()
    ctl = FixationController(list(range(n_layers)), 4, 0.125, focal, 0.05, warmup, 300, 256, 1, "cpu", ops=rec)
    q = [torch.zeros(1)] * n_layers
    have_last = False
    for t in range(1, steps + 1):
        rec.calls.clear()
        trace = ctl.step(t, _BATCH, q, q)
        plan = plan_step(t, n_layers, focal, warmup, have_last)
        assert [tuple(a) for a in plan.actions] == trace, (t, trace)
        # the calls behind each mode
        expect = []
        for layer, mode, src in trace:
            if mode == "full":
                expect.append("dense")
            elif mode == "full+select":
                expect += ["dense+score", "topk"]
            else:
                expect.append("sparse")
        assert [c[0] for c in rec.calls] == expect
        if plan.save_from is not None:
            have_last = True
            assert ctl.kept_from == plan.save_from          # the set kept for the next step
    return ctl


def test_hand_traced_four_layer_example():
    # C = {1, 3}, w = 2.  Step 3 (first after warm-up): no F_last -> layer 0 falls back to its own
    # top-k; step 4: layer 0 reuses F_last, 1 selects, 2 inherits 1's set, 3 selects, F_last = F_3.
    rec = Recorder()
    ctl = FixationController([0, 1, 2, 3], 4, 0.125, [1, 3], 0.05, 2, 300, 256, 1, "cpu", ops=rec)
    q = [torch.zeros(1)] * 4
    assert ctl.step(1, _BATCH, q, q) == [(0, "full", None), (1, "full", None), (2, "full", None), (3, "full", None)]
    ctl.step(2, _BATCH, q, q)
    assert ctl.step(3, _BATCH, q, q) == [(0, "full+select", None), (1, "full+select", None), (2, "pruned", 1),
                                       (3, "full+select", None)]
    assert ctl.step(4, _BATCH, q, q) == [(0, "pruned", "F_last"), (1, "full+select", None), (2, "pruned", 1),
                                       (3, "full+select", None)]
    assert ctl.kept_from == 3


@pytest.mark.parametrize("n_layers,focal,warmup", [
    (28, (2, 14), 4), (28, (0, 9, 20), 0), (6, (5,), 1), (1, (0,), 0), (36, (3, 11, 30), 10),
])
def test_schedule_matches_algorithm_1_for_many_steps(n_layers, focal, warmup):
    _run(n_layers, focal, warmup, warmup + 5)


def test_first_topk_is_cold_and_later_ones_are_warm_started():
    rec = Recorder()
    ctl = FixationController([0, 1, 2], 4, 0.125, [1], 0.05, 0, 300, 256, 1, "cpu", ops=rec)
    q = [torch.zeros(1)] * 3
    ctl.step(1, _BATCH, q, q)
    assert [c for c in rec.calls if c[0] == "topk"] == [("topk", False), ("topk", True)]
    rec.calls.clear()
    ctl.step(2, _BATCH, q, q)
    assert [c for c in rec.calls if c[0] == "topk"] == [("topk", True)]


def test_focal_gap_and_range_are_validated():
    mk = lambda focal, gap: FixationController(list(range(28)), 4, 0.1, focal, 0.05, 4, 300, 256, 1, "cpu",
                                               focal_gap=gap, ops=Recorder())
    mk((2, 14), 8)
    with pytest.raises(ValueError):
        mk((2, 10), 8)             # |i - j| must exceed the gap
    with pytest.raises(ValueError):
        mk((), 1)
    with pytest.raises(ValueError):
        mk((28,), 1)
    with pytest.raises(ValueError):
        plan_step(5, 4, (), 2, True)


def test_graph_replay_switch_brackets_the_step_s_calls():
    class Tuned(Recorder):
        def set_tuning(self, key, value):
            self.calls.append(("tune", key, value))
    rec = Tuned()
    ctl = FixationController([0, 1, 2], 4, 0.125, [1], 0.05, 0, 300, 256, 1, "cpu", ops=rec)
    q = [torch.zeros(1)] * 3
    ctl.step(1, _BATCH, q, q)
    assert not [c for c in rec.calls if c[0] == "tune"]
    rec.calls.clear()
    ctl.graph_replay = True
    ctl.step(2, _BATCH, q, q)
    assert rec.calls[0] == ("tune", "graph_replay", 1) and rec.calls[-1] == ("tune", "graph_replay", 0)
    assert len([c for c in rec.calls if c[0] == "tune"]) == 2

