"""Focal Layer Selection (Sec. 3.1.1, first block of Alg. 1): the oracle's transcription pinned
by hand-worked cases and by the properties the greedy rule implies; the library's host routine
against the oracle; the controller's warm-up profiling against a recorder."""
import ctypes
import itertools

import numpy as np
import pytest
import torch

from oracle.controller import select_focal_layers
import paper_2605_17447_amd as fo
from paper_2605_17447_amd import binding as fb
from paper_2605_17447_amd.binding import SeqBatch
from paper_2605_17447_amd.controller import FixationController

# geometry of three sequences; the recorder never looks inside, the controller reads its maxima
_BATCH = SeqBatch.from_lists([300, 280, 260], [10, 10, 10], [256, 256, 200], "cpu")


def test_hand_worked_cases():
    # 10 layers, mean ratios below; budget floor(0.3 * 10) = 3
    mean = [0.10, 0.50, 0.48, 0.05, 0.30, 0.47, 0.02, 0.40, 0.01, 0.45]
    # ranked: 1 (.50), 2 (.48), 5 (.47), 9 (.45), 7 (.40), 4 (.30), ...
    assert select_focal_layers([mean], 0.3, 0) == [1, 2, 5]            # gap 0: |i-j| > 0 always holds
    assert select_focal_layers([mean], 0.3, 1) == [1, 5, 9]            # 2 is next to 1; 5 ok; 9 ok
    assert select_focal_layers([mean], 0.3, 3) == [1, 5, 9]            # |5-1| = 4 > 3, |9-5| = 4 > 3
    assert select_focal_layers([mean], 0.3, 4) == [1, 9]               # 2, 5 within 4 of 1; 9 ok; the rest within 4 of 1 or 9
    assert select_focal_layers([mean], 0.1, 1) == [1]
    assert select_focal_layers([mean], 0.05, 1) == []                  # floor(0.5) = 0 focal layers
    # the mean runs over the warm-up steps: layer 0 wins only on average
    assert select_focal_layers([[0.9, 0.5, 0.1], [0.1, 0.4, 0.1], [0.5, 0.45, 0.1]], 0.34, 0) == [0]
    # ... and over the batch
    per_seq = np.array([[[0.2, 0.8], [0.6, 0.3], [0.1, 0.1]]])          # [1 step][3 layers][2 sequences]
    assert select_focal_layers(per_seq, 0.34, 0) == [0]                 # means 0.5, 0.45, 0.1
    # equal means: the lower layer is ranked first
    assert select_focal_layers([[0.3, 0.3, 0.3, 0.3]], 0.5, 1) == [0, 2]
    # rho * L a hair below an integer still counts (0.3 * 10 = 2.9999999999999996)
    assert len(select_focal_layers([list(np.linspace(1, 0, 10))], 0.3, 0)) == 3


@pytest.mark.parametrize("seed", range(20))
def test_greedy_properties(seed):
    rng = np.random.default_rng(seed)
    L, w = int(rng.integers(2, 40)), int(rng.integers(1, 6))
    r = rng.random((w, L))
    rho, gap = float(rng.choice([0.1, 0.2, 0.34, 0.5, 1.0])), int(rng.integers(0, 5))
    C = select_focal_layers(r, rho, gap)
    budget = int(np.floor(rho * L + 1e-9))
    mean = r.mean(axis=0)
    assert len(C) <= budget and C == sorted(set(C))
    assert all(abs(a - b) > gap for a, b in itertools.combinations(C, 2))
    if budget >= 1:
        assert int(np.argmax(mean)) in C                               # the best layer is always taken
    # a layer left out either met a full budget or lies within the gap of a better layer that was taken
    ranked = sorted(range(L), key=lambda i: (-mean[i], i))
    taken = []
    for i in ranked:
        blocked = any(abs(i - j) <= gap for j in taken)
        if i in C:
            assert not blocked and len(taken) < budget
            taken.append(i)
        else:
            assert blocked or len(taken) >= budget


@pytest.mark.parametrize("seed", range(25))
def test_library_routine_matches_the_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    w, L, B = int(rng.integers(1, 5)), int(rng.integers(1, 50)), int(rng.integers(1, 5))
    r = rng.random((w, L, B)).astype(np.float32)
    if seed % 4 == 0:
        r = np.round(r * 4) / 4                                        # many exact ties
    rho, gap = float(rng.choice([0.0, 0.1, 0.3, 0.5, 1.0])), int(rng.integers(0, 6))
    assert fb.select_focal_layers(r, rho, gap) == select_focal_layers(r, rho, gap)


def test_library_routine_rejects_bad_arguments():
    lib = fo.load_library()
    r = np.ones((2, 3, 1), np.float32)
    out = np.zeros(3, np.int32)
    n = ctypes.c_int32(0)
    call = lambda *a: lib.fastocr_select_focal_layers(*a)
    ok = (r.ctypes.data, 2, 3, 1, ctypes.c_double(0.5), 1, out.ctypes.data, ctypes.byref(n))
    assert call(*ok) == 0 and n.value == 1
    assert call(None, 2, 3, 1, ctypes.c_double(0.5), 1, out.ctypes.data, ctypes.byref(n)) == -1
    assert call(r.ctypes.data, 0, 3, 1, ctypes.c_double(0.5), 1, out.ctypes.data, ctypes.byref(n)) == -1
    assert call(r.ctypes.data, 2, 3, 1, ctypes.c_double(1.5), 1, out.ctypes.data, ctypes.byref(n)) == -1
    assert call(r.ctypes.data, 2, 3, 1, ctypes.c_double(0.5), -1, out.ctypes.data, ctypes.byref(n)) == -1
    bad = r.copy(); bad[0, 0, 0] = np.nan
    assert call(bad.ctypes.data, 2, 3, 1, ctypes.c_double(0.5), 1, out.ctypes.data, ctypes.byref(n)) == -1


class _Recorder:
    def __init__(self, chosen):
        self.calls, self.chosen = [], chosen

    def keep_count(self, n, tau):
        return max(1, int(n * tau))

    def workspace_bytes(self, *a, **k):
        return 256

    def dense_decode_attn(self, *a, **k):
        self.calls.append("dense")

    def focal_attn_score(self, cache, batch, q, scale, out, scores, ws, img_mass=None, **k):
        self.calls.append(("dense+score", img_mass is not None))

    def topk_fixation(self, *a, **k):
        self.calls.append("topk")

    def focal_attn_score_topk(self, *a, img_mass=None, **k):
        # a selecting layer is one call: full attention, scores and their top-k
        self.calls.append(("dense+score", img_mass is not None))
        self.calls.append("topk")

    def sparse_decode_attn(self, *a, **k):
        self.calls.append("sparse")

    def select_focal_layers(self, ratios, rho, gap):
        self.calls.append(("select", tuple(ratios.shape), rho, gap))
        return self.chosen


def test_controller_profiles_during_warm_up_and_then_uses_the_chosen_set():
    rec = _Recorder([1, 3])
    ctl = FixationController([0, 1, 2, 3], 4, 0.125, None, 0.05, 2, 300, 256, 3, "cpu", focal_gap=1, ops=rec,
                             focal_ratio=0.5)
    q = [torch.zeros(1)] * 4
    with pytest.raises(RuntimeError):
        ctl.step(3, _BATCH, q, q)                       # selection has not happened yet
    ctl.step(1, _BATCH, q, q)
    assert rec.calls == [("dense+score", True)] * 4 and ctl.focal is None
    rec.calls.clear()
    ctl.step(2, _BATCH, q, q)
    assert rec.calls[-1] == ("select", (2, 4, 3), 0.5, 1) and ctl.focal == [1, 3]
    rec.calls.clear()
    trace = ctl.step(3, _BATCH, q, q)
    assert [m for _, m, _ in trace] == ["full+select", "full+select", "pruned", "full+select"]
    with pytest.raises(ValueError):
        FixationController([0, 1], 4, 0.1, None, 0.05, 0, 300, 256, 1, "cpu", ops=rec)     # no warm-up to profile
    with pytest.raises(ValueError):
        FixationController([0, 1], 4, 0.1, None, 0.05, 2, 300, 256, 1, "cpu", ops=rec, focal_ratio=0.1)
