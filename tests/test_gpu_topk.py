"""GPU parity of the top-k selection on its own: identical fp32 scores go to the kernel and to
the oracle's full sort, so the index sets must agree bit for bit, ties included; the previous
step's set (warm start) must never change the result."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_17447_amd as fo
from paper_2605_17447_amd import binding as fb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_topk(scores_np, vis_len, tau, prev=None, kmax=None, inplace=False):
    B, W = scores_np.shape
    sc = torch.from_numpy(scores_np).to(DEV)
    batch = fo.SeqBatch.from_lists([int(n) + 3 for n in vis_len], [1] * B, [int(n) for n in vis_len], DEV)
    batch.max_vis_len = W
    batch.max_seq_len = W + 3
    kmax = kmax or max(1, fo.keep_count(W, tau))
    ws_bytes = fo.workspace_bytes(fb.OP_TOPK_FIXATION, None, batch, 0, kmax)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=DEV)
    if prev is not None:
        pidx = torch.from_numpy(prev[0]).to(DEV).contiguous()
        pcnt = torch.from_numpy(prev[1]).to(DEV)
    else:
        pidx = pcnt = None
    if inplace:
        idx, cnt = pidx, pcnt
    else:
        idx = torch.full((B, kmax), -5, dtype=torch.int32, device=DEV)
        cnt = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    fo.topk_fixation(sc, batch, tau, idx, cnt, ws, pidx, pcnt)
    return idx.cpu().numpy(), cnt.cpu().numpy()


def expect(scores_np, vis_len, tau):
    return [oracle.topk(scores_np[b, : vis_len[b]], oracle.keep_count(int(vis_len[b]), tau))
            for b in range(scores_np.shape[0])]


def assert_same(idx, cnt, want, what=""):
    for b, w in enumerate(want):
        assert cnt[b] == len(w), f"{what} b={b}: count {cnt[b]} != {len(w)}"
        assert np.array_equal(idx[b, : len(w)], w), f"{what} b={b}: index set differs"


def make_scores(rng, B, W, kind):
    if kind == "softmax":           # the shape real scores have: positive, tiny, a narrow exponent range
        x = rng.normal(size=(B, W)) * 0.5
        s = np.exp(x) / np.exp(x).sum(axis=1, keepdims=True)
    elif kind == "ties":            # few distinct values -> long runs of exact ties across the threshold
        s = rng.integers(0, 7, size=(B, W)) / 64.0
    elif kind == "signed":          # negative values, zeros, infinities: the key transform must order them
        s = rng.normal(size=(B, W))
        s[:, ::17] = 0.0
        s[:, 5::97] = -0.0
        s[0, 3 % W] = np.inf
        s[0, 7 % W] = -np.inf
    elif kind == "const":
        s = np.full((B, W), 0.125)
    elif kind == "cluster":         # a dense cluster a few thousand ulps wide under a few far outliers: the
        # select has to narrow its window several times, down to single key values (with repeats)
        s = (1.0 + rng.integers(0, 3000, size=(B, W)) * 2.0 ** -23).astype(np.float32)
        s[:, ::1000] = 100.0
        s[1 % B] = (1.0 + rng.integers(0, 200000, size=W) * 2.0 ** -23).astype(np.float32)     # wider: ends in a ranked bin
        s[1 % B, ::777] = 1.0e6
    return s.astype(np.float32)


@pytest.mark.parametrize("kind", ["softmax", "ties", "signed", "const", "cluster"])
@pytest.mark.parametrize("W", [1, 5, 64, 1000, 4096, 6000, 8192, 16384, 20000])
def test_cold_topk_is_bit_exact(kind, W):
    rng = np.random.default_rng(W * 3 + len(kind))
    B = 3
    s = make_scores(rng, B, W, kind)
    vis_len = [W, max(1, W // 2 + 1), max(1, W - 3)]
    for tau in (0.02, 0.05, 0.5, 1.0):
        idx, cnt = run_topk(s, vis_len, tau)
        assert_same(idx, cnt, expect(s, vis_len, tau), f"{kind} W={W} tau={tau}")


@pytest.mark.parametrize("W", [300, 4096, 16384, 20000])
def test_nan_scores_order_above_every_number(W):
    """A score the scoring launch could not finish is a (positive, quiet) NaN; the select takes those
    first, like the largest numbers.  The oracle's sort has no place for a NaN, so it gets the same
    rows with +inf in their place (no other infinity is present)."""
    rng = np.random.default_rng(W)
    s = make_scores(rng, 3, W, "softmax")
    vis_len = [W, W // 2 + 1, W - 3]
    for b in range(3):
        s[b, rng.choice(vis_len[b], 3, replace=False)] = np.nan
    stand_in = np.where(np.isnan(s), np.float32(np.inf), s)
    for tau in (0.02, 0.5):
        idx, cnt = run_topk(s, vis_len, tau)
        assert_same(idx, cnt, expect(stand_in, vis_len, tau), f"NaN W={W} tau={tau}")


def test_scores_beyond_the_lds_key_capacity_use_the_workspace():
    rng = np.random.default_rng(1)
    s = make_scores(rng, 2, 40000, "softmax")
    s2 = make_scores(rng, 2, 40000, "ties")
    for arr in (s, s2):
        idx, cnt = run_topk(arr, [40000, 33333], 0.05)
        assert_same(idx, cnt, expect(arr, [40000, 33333], 0.05), "N=40000")


def test_warm_start_never_changes_the_result():
    rng = np.random.default_rng(2)
    B, W, tau = 4, 16384, 0.05
    vis_len = [16384, 16384, 9000, 12345]
    for kind in ("softmax", "ties"):
        s = make_scores(rng, B, W, kind)
        want = expect(s, vis_len, tau)
        kmax = fo.keep_count(W, tau)
        k_b = [len(w) for w in want]

        def pack(rows):
            a = np.zeros((B, kmax), np.int32)
            for b, r in enumerate(rows):
                a[b, : len(r)] = r
            return a

        cnts = np.array(k_b, np.int32)
        # (a) a good previous set: the top-k of slightly perturbed scores (a fixation that moved a little)
        s_prev = (s * (1 + 0.05 * rng.normal(size=s.shape))).astype(np.float32)
        good = pack(expect(s_prev, vis_len, tau))
        # (b) a stale set: k random distinct tokens (candidate list overflows -> full select)
        stale = pack([np.sort(rng.choice(vis_len[b], k_b[b], replace=False)) for b in range(B)])
        # (c) the answer itself
        exact = pack(want)
        # (d) malformed sets: unsorted, duplicate, out of range, wrong count -> ignored
        unsorted_ = exact.copy(); unsorted_[:, [0, 1]] = unsorted_[:, [1, 0]]
        dup = exact.copy(); dup[:, 1] = dup[:, 0]
        oor = exact.copy(); oor[:, 0] = -3
        oor2 = exact.copy()
        for b in range(B):
            oor2[b, k_b[b] - 1] = vis_len[b]
        for name, prev, pc in [("good", good, cnts), ("stale", stale, cnts), ("exact", exact, cnts),
                               ("unsorted", unsorted_, cnts), ("dup", dup, cnts), ("neg", oor, cnts),
                               ("past-end", oor2, cnts), ("wrong-count", exact, cnts - 1),
                               ("zero-count", exact, np.zeros(B, np.int32))]:
            idx, cnt = run_topk(s, vis_len, tau, prev=(prev, pc), kmax=kmax)
            assert_same(idx, cnt, want, f"{kind} prev={name}")
        # in place: the previous set's buffers receive the new set
        idx, cnt = run_topk(s, vis_len, tau, prev=(good.copy(), cnts.copy()), kmax=kmax, inplace=True)
        assert_same(idx, cnt, want, f"{kind} in-place")


def test_rows_beyond_the_count_are_left_alone_and_pitch_may_exceed_k():
    rng = np.random.default_rng(3)
    s = make_scores(rng, 2, 500, "softmax")
    idx, cnt = run_topk(s, [500, 100], 0.1, kmax=77)
    assert_same(idx, cnt, expect(s, [500, 100], 0.1))
    assert np.all(idx[0, 50:] == -5) and np.all(idx[1, 10:] == -5)


def test_warm_start_with_more_kept_tokens_than_threads_and_few_kept_tokens():
    """Keep ratios above 1/16 (the previous set is longer than the workgroup, and the bound from the
    threads' own maxima does not apply) and a very small one."""
    rng = np.random.default_rng(4)
    B, W = 3, 16384
    vis_len = [16384, 10000, 16001]
    for kind in ("softmax", "cluster"):
        s = make_scores(rng, B, W, kind)
        for tau in (0.25, 0.004):
            want = expect(s, vis_len, tau)
            kmax = fo.keep_count(W, tau)
            s_prev = (s * (1 + 0.02 * rng.normal(size=s.shape))).astype(np.float32)
            prev = np.zeros((B, kmax), np.int32)
            for b, r in enumerate(expect(s_prev, vis_len, tau)):
                prev[b, : len(r)] = r
            cnts = np.array([len(w) for w in want], np.int32)
            idx, cnt = run_topk(s, vis_len, tau, prev=(prev, cnts), kmax=kmax)
            assert_same(idx, cnt, want, f"{kind} tau={tau} warm")
            idx, cnt = run_topk(s, vis_len, tau, kmax=kmax)
            assert_same(idx, cnt, want, f"{kind} tau={tau} cold")


def test_score_rows_that_do_not_start_on_16_bytes():
    """A view into a larger buffer: rows start 4 bytes past a 16-byte boundary (the kernel then
    reads score by score), with and without a previous set."""
    rng = np.random.default_rng(5)
    B, W, tau = 2, 4096, 0.05
    s = make_scores(rng, B, W, "softmax")
    vis_len = [4096, 3000]
    want = expect(s, vis_len, tau)
    big = torch.zeros(B * W + 1, dtype=torch.float32, device=DEV)
    sc = big[1:].view(B, W)
    sc.copy_(torch.from_numpy(s))
    assert sc.data_ptr() % 16 == 4
    batch = fo.SeqBatch.from_lists([n + 3 for n in vis_len], [1] * B, vis_len, DEV)
    batch.max_vis_len = W
    batch.max_seq_len = W + 3
    kmax = fo.keep_count(W, tau)
    ws = torch.empty(256, dtype=torch.uint8, device=DEV)
    idx = torch.full((B, kmax), -5, dtype=torch.int32, device=DEV)
    cnt = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    fo.topk_fixation(sc, batch, tau, idx, cnt, ws)
    assert_same(idx.cpu().numpy(), cnt.cpu().numpy(), want, "unaligned cold")
    fo.topk_fixation(sc, batch, tau, idx, cnt, ws, idx, cnt)
    assert_same(idx.cpu().numpy(), cnt.cpu().numpy(), want, "unaligned warm, in place")
