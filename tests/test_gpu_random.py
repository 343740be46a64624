"""GPU parity on seeded random small problems: shapes, lengths, keep ratios, layouts, paging and
launch-shape overrides drawn at random, every call checked against the oracle as in
test_gpu_parity.full_check.  The draws are fixed by the seeds below."""
import numpy as np
import pytest
import torch

import fastocr_synth as fs
from paper_2605_17447_amd import binding as fb
from util import TinyCase

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DEV, GpuProblem, problem_from_case
    from test_gpu_parity import full_check

MFMA_HEADS = [(28, 4), (64, 8), (16, 1), (4, 4), (6, 2), (8, 1), (32, 8), (16, 2), (12, 4), (3, 1), (16, 16), (10, 2)]
PLAIN_SHAPES = [(4, 1, 64), (6, 3, 32), (8, 8, 16), (7, 1, 40), (4, 2, 64), (8, 2, 96), (12, 4, 256), (5, 5, 128), (32, 2, 64), (34, 2, 64)]
TAUS = [0.05, 0.02, 0.1, 0.25, 0.004, 1.0, 0.0, 0.5]


def _draw(rng):
    """One random problem description (no tensors yet)."""
    mfma = rng.random() < 0.7
    if mfma:
        (Hq, Hkv), d, dtype = MFMA_HEADS[rng.integers(len(MFMA_HEADS))], 128, "bf16"
    else:
        Hq, Hkv, d = PLAIN_SHAPES[rng.integers(len(PLAIN_SHAPES))]
        dtype = "bf16" if rng.random() < 0.4 else "f32"
    B = int(rng.integers(1, 7))
    big = mfma and rng.random() < 0.5

    def n_image():
        r = rng.random()
        if r < 0.1:
            return 0
        if r < 0.3:
            return int(rng.integers(1, 40))
        return int(rng.integers(1, 5000 if big else 1400))

    n_vis = [n_image() for _ in range(B)]
    pre = [int(rng.integers(0, 90)) if rng.random() < 0.8 else 0 for _ in range(B)]
    post = [int(rng.integers(0, 300)) if rng.random() < 0.8 else 0 for _ in range(B)]
    if rng.random() < 0.1:                               # an empty sequence
        j = int(rng.integers(B))
        n_vis[j] = pre[j] = post[j] = 0
    tune = {}
    if rng.random() < 0.5:
        for key in ("splits_score", "splits_dense", "splits_sparse"):
            tune[key] = int(rng.integers(0, 7))
    if rng.random() < 0.3:
        tune["attn_merge"] = int(rng.integers(0, 3))
    if rng.random() < 0.3:
        tune["attn_waves"] = int([4, 8][rng.integers(2)])
    return dict(mfma=mfma, Hq=Hq, Hkv=Hkv, d=d, dtype=dtype, B=B, n_vis=n_vis, pre=pre, post=post,
                tau=float(TAUS[rng.integers(len(TAUS))]), tune=tune,
                layout="bshd" if rng.random() < 0.3 else "bhsd", paged=mfma and rng.random() < 0.25,
                # keys and queries up to three times the workload's spread, for every dtype (logits near 30)
                spread=float([1.0, 1.0, 3.0, 0.3][rng.integers(4)]),
                seed=int(rng.integers(1 << 30)))


@pytest.mark.parametrize("seed", range(4))
def test_random_small_problems(seed):
    rng = np.random.default_rng(1000 + seed)
    done = 0
    timeouts_before = fb.exchange_timeouts()          # counted since the library was loaded
    for n in range(40):
        c = _draw(rng)
        what = f"random seed {seed} case {n}: " + ", ".join(f"{k}={v}" for k, v in c.items())
        try:
            for key, value in c["tune"].items():
                fb.set_tuning(key, value)
            if c["paged"]:
                lo = int(rng.integers(64, 1500))
                hi = lo + int(rng.integers(1, 3000))
                page = int([16, 64, 128][rng.integers(3)])
                wl = fs.config(5, batch=c["B"], steps=8, n_visual=(lo, hi), grid_w=(16, 50), text_prefix=(3, 300),
                               page_tokens=page)
                bt = fs.make_batch(wl, seed=c["seed"], device=DEV)
                t = int(rng.integers(1, 9))
                q = fs.queries_for_step(bt, t, [x[t - 1] for x in fs.centres(bt)])
                p = GpuProblem(bt.k, bt.v, q, bt.seq_len(t), bt.vis_start, bt.n_vis, wl.head_dim ** -0.5,
                               block_table=bt.block_table)
                full_check(p, c["tau"] if c["tau"] > 0 else 0.05, what + f" paged {lo}..{hi} page {page} step {t}")
            else:
                case = TinyCase(seed=c["seed"], B=c["B"], Hq=c["Hq"], Hkv=c["Hkv"], d=c["d"], n_vis=c["n_vis"],
                                pre=c["pre"], post=c["post"], dtype=c["dtype"], spread=c["spread"])
                if int(case.seq_len.max()) == 0:
                    continue
                full_check(problem_from_case(case, c["layout"]), c["tau"], what)
            done += 1
        finally:
            for key in ("splits_score", "splits_dense", "splits_sparse"):
                fb.set_tuning(key, 0)
            fb.set_tuning("attn_merge", 1)
            fb.set_tuning("attn_waves", 4)
    assert done >= 30
    assert fb.exchange_timeouts() == timeouts_before
