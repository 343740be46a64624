"""The runs the workload configurations describe, at their full shapes, against the oracle along
the way: configuration 2's 512-step chain in which every step's focal token set bounds the next
step's selection in place (Cross-Step Fixation Reuse, Sec. 3.2), and decode steps of the 28-layer
stacks of configurations 3 and 5 through the step controller (Alg. 1: warm-up, the fallback step,
Cross-Layer Propagation, layer 0 on the previous step's set)."""
import numpy as np
import pytest
import torch

import fastocr_synth as fs
import oracle
from oracle.controller import plan_step
import paper_2605_17447_amd as fo
from paper_2605_17447_amd import binding as fb

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DEV, GpuProblem, check_out, check_scores, check_set_valid
    from test_gpu_parity import full_check


def test_config1_on_a_hundred_seeds():
    wl = fs.config(1)
    for seed in range(6, 106):
        bt = fs.make_batch(wl, seed=fs.BASE_SEED + 31 * seed, device=DEV)
        q = fs.queries_for_step(bt, 1, [x[0] for x in fs.centres(bt)])
        p = GpuProblem(bt.k, bt.v, q, bt.seq_len(1), bt.vis_start, bt.n_vis, wl.head_dim ** -0.5)
        full_check(p, 0.05, f"config1 seed {seed}")


def test_config2_whole_run_with_warm_started_sets_in_place():
    """512 decode steps on one layer: 4 warm-up steps of full attention, then score -> top-k ->
    pruned attention at every step, the set refreshed in place with itself as the previous set.
    Every step must keep 205 tokens; every 16th step is compared with the oracle (scores, the set
    bit for bit on the path's own scores and as a valid set on the oracle's, the output)."""
    wl = fs.config(2)
    tau, w = 0.05, wl.warmup
    bt = fs.make_batch(wl, device=DEV)
    cs = fs.centres(bt)
    B, Hq, d = wl.batch, wl.n_q_heads, wl.head_dim
    scale = float(np.float32(d ** -0.5))
    cache = fo.KvCache(bt.k, bt.v)
    oc = oracle.Cache.from_bhsd(fs.to_oracle_array(bt.k), fs.to_oracle_array(bt.v))
    max_seq, max_vis = max(bt.seq_len(wl.steps)), max(bt.n_vis)
    seq_len = torch.tensor(bt.seq_len(1), dtype=torch.int32, device=DEV)
    batch = fo.SeqBatch(seq_len, torch.tensor(bt.vis_start, dtype=torch.int32, device=DEV),
                        torch.tensor(bt.n_vis, dtype=torch.int32, device=DEV), max_seq, max_vis)
    kmax = fo.keep_count(max_vis, tau)
    assert kmax == 205
    ws = torch.empty(max(fo.workspace_bytes(op, cache, batch, Hq, kmax) for op in range(5)), dtype=torch.uint8, device=DEV)
    scores = torch.zeros((B, max_vis), dtype=torch.float32, device=DEV)
    idx = torch.full((B, kmax), -1, dtype=torch.int32, device=DEV)
    cnt = torch.zeros((B,), dtype=torch.int32, device=DEV)
    out = torch.zeros((B, Hq, d), dtype=torch.bfloat16, device=DEV)
    counts = torch.zeros((wl.steps + 1, B), dtype=torch.int32, device=DEV)
    timeouts_before = fb.exchange_timeouts()
    checked, prev_set, overlaps = 0, None, []
    for t in range(1, wl.steps + 1):
        q = fs.queries_for_step(bt, t, [c[t - 1] for c in cs])
        args = (oc, bt.seq_len(t), bt.vis_start, bt.n_vis, fs.to_oracle_array(q), scale)
        if t <= w:
            fo.dense_decode_attn(cache, batch, q, scale, out, ws)
            check_out(out, oracle.decode_attn(*args)[0], f"warm-up step {t}")
        else:
            fo.focal_score(cache, batch, q, scale, scores, ws)
            warm = t > w + 1
            fo.topk_fixation(scores, batch, tau, idx, cnt, ws, prev_idx=idx if warm else None, prev_cnt=cnt if warm else None)
            fo.sparse_decode_attn(cache, batch, q, scale, idx, cnt, out, ws)
            counts[t].copy_(cnt)
            if t % 16 == 0 or t in (w + 1, w + 2, wl.steps):
                ref_sc, _, _ = oracle.focal_score(*args)
                check_scores(scores, ref_sc, bt.n_vis, f"step {t} scores")
                sc_h, idx_h, cnt_h = scores.cpu().numpy(), idx.cpu().numpy(), cnt.cpu().numpy()
                for b in range(B):
                    check_set_valid(idx_h[b], int(cnt_h[b]), ref_sc[b], kmax, f"step {t} set")
                    assert np.array_equal(idx_h[b, :kmax], oracle.topk(sc_h[b], kmax)), f"step {t}: set differs on identical scores"
                ref, _ = oracle.decode_attn(*args, idx_h, cnt_h)
                check_out(out, ref, f"step {t} pruned attention")
                if prev_set is not None and prev_set[0] == t - 1:
                    overlaps.append(len(np.intersect1d(prev_set[1], idx_h[0, :kmax])) / kmax)
                checked += 1
            if (t + 1) % 16 == 0:
                prev_set = (t, idx[0, :kmax].cpu().numpy().copy())
        seq_len.add_(1)
    torch.cuda.synchronize()
    assert torch.all(counts[w + 1:] == kmax), "every step after warm-up keeps ceil(0.05 * 4096) = 205 tokens"
    assert checked >= 32
    assert fb.exchange_timeouts() == timeouts_before
    # the warm start had something to work with: consecutive sets share tokens
    assert overlaps and min(overlaps) > 0.05


def _oracle_cache(x):
    k, v = fs.to_oracle_array(x.k), fs.to_oracle_array(x.v)
    if x.block_table is None:
        return oracle.Cache.from_bhsd(k, v)
    n_pages, H, pt, dd = k.shape
    return oracle.Cache(k, v, H, dd, stride_token=dd, stride_head=pt * dd, page_tokens=pt,
                        stride_page=H * pt * dd, block_table=x.block_table.cpu().numpy())


@pytest.mark.parametrize("cfg", [3, 5])
def test_28_layer_stack_steps_at_full_shape(cfg):
    """Configuration 3 (batch 8, N = 4096) and configuration 5 (batch 32, ragged image spans up to 16384
    tokens, paged) as 28-layer stacks with focal layers {2, 14}, through the step controller: the
    warm-up steps, the fallback step (layer 0 selects for itself) and a steady-state step in which
    layer 0 attends the previous step's set.  The schedule of every step is the oracle controller's;
    at the fallback and steady-state steps every selecting layer (output, scores, set) and layers 0, 1,
    3, 13, 15 and 27 (pruned by F_last, by layer 2's set and by layer 14's) are compared with the oracle."""
    wl = fs.config(cfg, steps=8)
    L, focal, w, tau = wl.n_layers, wl.focal_layers, wl.warmup, 0.05
    assert L == 28 and tuple(focal) == (2, 14) and w == 4
    bts = [fs.make_batch(wl, device=DEV, layer=l) for l in range(L)]
    bt = bts[0]
    cs = fs.centres(bt)
    B, Hq, d = wl.batch, wl.n_q_heads, wl.head_dim
    scale = float(np.float32(d ** -0.5))
    caches = [fo.KvCache(x.k, x.v, "bhsd", x.block_table) for x in bts]
    max_seq, max_vis = max(bt.seq_len(wl.steps)), max(bt.n_vis)
    ctl = fo.FixationController(caches, Hq, scale, focal, tau, w, max_seq, max_vis, B, DEV, focal_gap=wl.focal_gap)
    sampled = (0, 1, 3, 13, 15, 27)
    have_last, kept_by = False, {}
    timeouts_before = fb.exchange_timeouts()
    for t in range(1, w + 3):
        seq_len = bt.seq_len(t)
        batch = fo.SeqBatch.from_lists(seq_len, bt.vis_start, bt.n_vis, DEV)
        qs = [fs.queries_for_step(bts[l], t, [c[t - 1] for c in cs]) for l in range(L)]
        outs = [torch.zeros_like(q) for q in qs]
        picked = {}
        trace = ctl.step(t, batch, qs, outs,
                         on_select=lambda l, sc, idx, cnt: picked.__setitem__(l, (sc.clone(), idx.clone(), cnt.clone())))
        torch.cuda.synchronize()
        plan = plan_step(t, L, focal, w, have_last)
        assert [tuple(a) for a in plan.actions] == trace, f"step {t}: schedule differs"
        if t <= w:
            # warm-up: full attention everywhere; two layers are enough to pin it at this shape
            for l in ((0, 27) if t == 1 else (14,)):
                args = (_oracle_cache(bts[l]), seq_len, bt.vis_start, bt.n_vis, fs.to_oracle_array(qs[l]), scale)
                check_out(outs[l], oracle.decode_attn(*args)[0], f"config {cfg} warm-up step {t} layer {l}")
            continue
        if t == w + 1:
            assert plan.actions[0].mode == "full+select"           # nothing survives the warm-up: layer 0 selects
        else:
            assert plan.actions[0] == (0, "pruned", "F_last")
        # the sets this step's layers attend: F_last is what the deepest focal layer left at the previous step
        sets = {"F_last": kept_by.get(max(focal))}
        for action in plan.actions:
            l = action.layer
            if action.mode == "full+select":
                args = (_oracle_cache(bts[l]), seq_len, bt.vis_start, bt.n_vis, fs.to_oracle_array(qs[l]), scale)
                check_out(outs[l], oracle.decode_attn(*args)[0], f"config {cfg} step {t} layer {l} full")
                ref_sc, _, _ = oracle.focal_score(*args)
                ref_idx, ref_cnt = oracle.topk_fixation(ref_sc, bt.n_vis, tau)
                check_scores(picked[l][0], ref_sc, bt.n_vis, f"config {cfg} step {t} layer {l} scores")
                sc_h, idx_h, cnt_h = (x.cpu().numpy() for x in picked[l])
                for b in range(B):
                    n = bt.n_vis[b]
                    check_set_valid(idx_h[b], int(cnt_h[b]), ref_sc[b, :n], int(ref_cnt[b]), f"config {cfg} step {t} layer {l} set b={b}")
                    assert np.array_equal(idx_h[b, : cnt_h[b]], oracle.topk(sc_h[b, :n], int(ref_cnt[b])))
                # the reference carries the (validated) set the path chose, so later layers attend the same tokens
                sets[l] = (idx_h.copy(), cnt_h.copy())
            elif l in sampled:
                idx_h, cnt_h = sets[action.set_from]
                args = (_oracle_cache(bts[l]), seq_len, bt.vis_start, bt.n_vis, fs.to_oracle_array(qs[l]), scale)
                ref, _ = oracle.decode_attn(*args, idx_h, cnt_h)
                check_out(outs[l], ref, f"config {cfg} step {t} layer {l} pruned by {action.set_from}")
        kept_by = {l: s for l, s in sets.items() if l != "F_last"}
        have_last = plan.save_from is not None
        assert ctl.kept_from == plan.save_from
    assert fb.exchange_timeouts() == timeouts_before
