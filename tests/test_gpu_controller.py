"""A small attention-only stack driven by the step controller on the GPU, against the same
stack evaluated layer by layer with the oracle following the oracle's reading of Algorithm 1:
warm-up steps, the fallback selection of the first step after warm-up, cross-layer propagation
of the kept set and its reuse by the layers before the first focal layer at the next step."""
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
    from gpu_util import DEV, check_out, check_scores, check_set_valid


@pytest.mark.parametrize("paged", [False, True])
def test_stack_follows_algorithm_1(paged):
    L, focal, warmup, tau, steps = 6, (1, 4), 2, 0.1, 6
    wl = fs.config(5 if paged else 3, batch=3, n_layers=L, focal_layers=focal, steps=steps, warmup=warmup,
                   n_visual=(700, 1100) if paged else (1024, 1024), grid_w=(24, 40) if paged else (32, 32),
                   text_prefix=(9, 60), page_tokens=64)
    bts = [fs.make_batch(wl, device=DEV, layer=l) for l in range(L)]
    bt = bts[0]
    cs = fs.centres(bt)
    B, Hq, d = wl.batch, wl.n_q_heads, wl.head_dim
    scale = float(np.float32(d ** -0.5))
    caches = [fo.KvCache(x.k, x.v, "bhsd", x.block_table) for x in bts]
    max_seq, max_vis = max(bt.seq_len(steps)), max(bt.n_vis)
    ctl = fo.FixationController(caches, Hq, scale, focal, tau, warmup, max_seq, max_vis, B, DEV, focal_gap=2)

    def oracle_cache(x):
        k, v = fs.to_oracle_array(x.k), fs.to_oracle_array(x.v)
        if x.block_table is None:
            return oracle.Cache.from_bhsd(k, v)
        n_pages, H, pt, dd = k.shape
        return oracle.Cache(k, v, H, dd, stride_token=dd, stride_head=pt * dd, page_tokens=pt,
                            stride_page=H * pt * dd, block_table=x.block_table.cpu().numpy())
    ocs = [oracle_cache(x) for x in bts]

    have_last = False
    kept = None                          # (idx, cnt) numpy: the set the reference pipeline carries
    for t in range(1, steps + 1):
        seq_len = bt.seq_len(t)
        batch = fo.SeqBatch.from_lists(seq_len, bt.vis_start, bt.n_vis, DEV)
        qs = [fs.queries_for_step(bts[l], t, [c[t - 1] for c in cs]) for l in range(L)]
        outs = [torch.zeros_like(q) for q in qs]
        picked = {}
        trace = ctl.step(t, batch, qs, outs,
                         on_select=lambda l, sc, idx, cnt: picked.__setitem__(l, (sc.clone(), idx.clone(), cnt.clone())))
        torch.cuda.synchronize()
        plan = plan_step(t, L, focal, warmup, have_last)
        assert [tuple(a) for a in plan.actions] == trace, f"step {t}: schedule differs"
        for action in plan.actions:
            l = action.layer
            args = (ocs[l], seq_len, bt.vis_start, bt.n_vis, fs.to_oracle_array(qs[l]), scale)
            if action.mode == "pruned":
                ref, _ = oracle.decode_attn(*args, kept[0], kept[1])
                check_out(outs[l], ref, f"step {t} layer {l} pruned")
                continue
            ref, _ = oracle.decode_attn(*args)
            check_out(outs[l], ref, f"step {t} layer {l} full")
            if action.mode == "full+select":
                ref_sc, _, _ = oracle.focal_score(*args)
                ref_idx, ref_cnt = oracle.topk_fixation(ref_sc, bt.n_vis, tau)
                sc, idx, cnt = (x.cpu().numpy() for x in picked[l])
                check_scores(picked[l][0], ref_sc, bt.n_vis, f"step {t} layer {l} scores")
                for b in range(B):
                    check_set_valid(idx[b], int(cnt[b]), ref_sc[b, : bt.n_vis[b]], int(ref_cnt[b]),
                                    f"step {t} layer {l} set b={b}")
                # the set is unique only up to ties within the tolerance: the reference carries the
                # (validated) set the GPU path chose, so that later layers attend the same tokens
                kept = (idx.copy(), cnt.copy())
        if plan.save_from is not None:
            have_last = True
            assert ctl.kept_from == plan.save_from


def test_focal_layers_are_chosen_from_the_warm_up_ratios():
    """Focal Layer Selection on the GPU path: layers differ in how much attention mass their
    queries put on the image (a per-layer gain on the fixation window), the controller records
    each layer's image-attention ratio during warm-up and picks the focal set; ratios and set
    must match the oracle's."""
    import dataclasses
    L, warmup, tau, rho, gap = 8, 3, 0.1, 0.4, 1
    gains = [0.6, 3.0, 2.0, 0.8, 1.0, 3.5, 0.7, 1.5]             # ranked: 5, 1, 2, 7, ... -> with gap 1: {1, 5, 7}
    base = fs.config(3, batch=2, n_layers=L, steps=warmup + 1, warmup=warmup, n_visual=(576, 576), grid_w=(24, 24),
                     text_prefix=(400, 400))
    bts = [fs.make_batch(dataclasses.replace(base, beta=g), device=DEV, layer=l) for l, g in enumerate(gains)]
    bt = bts[0]
    cs = fs.centres(bt)
    B, Hq, d = base.batch, base.n_q_heads, base.head_dim
    scale = float(np.float32(d ** -0.5))
    caches = [fo.KvCache(x.k, x.v) for x in bts]
    ctl = fo.FixationController(caches, Hq, scale, None, tau, warmup, max(bt.seq_len(warmup + 1)), max(bt.n_vis), B, DEV,
                                focal_gap=gap, focal_ratio=rho)
    ref = np.zeros((warmup, L, B))
    for t in range(1, warmup + 1):
        seq_len = bt.seq_len(t)
        batch = fo.SeqBatch.from_lists(seq_len, bt.vis_start, bt.n_vis, DEV)
        qs = [fs.queries_for_step(bts[l], t, [c[t - 1] for c in cs]) for l in range(L)]
        outs = [torch.zeros_like(q) for q in qs]
        ctl.step(t, batch, qs, outs)
        for l in range(L):
            oc = oracle.Cache.from_bhsd(fs.to_oracle_array(bts[l].k), fs.to_oracle_array(bts[l].v))
            _, _, mass = oracle.focal_score(oc, seq_len, bt.vis_start, bt.n_vis, fs.to_oracle_array(qs[l]), scale)
            ref[t - 1, l] = mass
    torch.cuda.synchronize()
    got = ctl.ratios.cpu().numpy()
    assert np.abs(got - ref).max() <= 2e-5, "image-attention ratios differ from the oracle"
    from oracle.controller import select_focal_layers
    want = select_focal_layers(ref, rho, gap)
    assert ctl.focal == want and len(want) == 3
    # the ranking is not an accident of noise: the chosen layers are those with the largest gains allowed by the gap
    assert want == [1, 5, 7]
    # and the next step runs with the chosen set
    t = warmup + 1
    batch = fo.SeqBatch.from_lists(bt.seq_len(t), bt.vis_start, bt.n_vis, DEV)
    qs = [fs.queries_for_step(bts[l], t, [c[t - 1] for c in cs]) for l in range(L)]
    trace = ctl.step(t, batch, qs, [torch.zeros_like(q) for q in qs])
    assert [tuple(a) for a in plan_step(t, L, want, warmup, False).actions] == trace


@pytest.mark.parametrize("form", [1, 2])
def test_a_captured_decode_step_replays_like_the_eager_one(form):
    """The calls allocate nothing and never synchronise, so a whole decode step of the
    controller can be captured in a HIP graph (launch-bound small shapes).  Every replay, with
    fresh queries and a longer sequence, must match the eager controller bit for bit; eager work
    and synchronisations sit between the replays.  form 2 forces the register-resident kernels
    (a captured launch keeps its barrier slot, which every replay must find clean again)."""
    fb.set_tuning("score_resident", form)
    fb.set_tuning("focal_fused", form)
    try:
        _captured_step_replays()
    finally:
        fb.set_tuning("score_resident", 1)
        fb.set_tuning("focal_fused", 1)


def test_a_captured_decode_step_with_the_graph_replay_hint():
    """The same with the controllers told that their steps are replayed from a graph (pruned attention over
    these short lists is then partials plus the merge kernel): eager and captured steps still agree bit for
    bit, because the hint, not the capture, decides the launch shapes."""
    _captured_step_replays(hint=True)


def _captured_step_replays(hint=False):
    L, focal, tau, steps = 5, (1, 3), 0.1, 10
    wl = fs.config(3, batch=2, n_layers=L, focal_layers=focal, steps=steps, warmup=0, n_visual=(1024, 1024),
                   grid_w=(32, 32), text_prefix=(30, 30))
    bts = [fs.make_batch(wl, device=DEV, layer=l) for l in range(L)]
    bt = bts[0]
    cs = fs.centres(bt)
    B, Hq, d = wl.batch, wl.n_q_heads, wl.head_dim
    scale = float(np.float32(d ** -0.5))
    caches = [fo.KvCache(x.k, x.v) for x in bts]
    max_seq, max_vis = max(bt.seq_len(steps)), max(bt.n_vis)
    mk = lambda: fo.FixationController(caches, Hq, scale, focal, tau, 0, max_seq, max_vis, B, DEV, focal_gap=1)
    eager, graphed = mk(), mk()
    eager.graph_replay = graphed.graph_replay = hint
    queries = lambda t: [fs.queries_for_step(bts[l], t, [c[t - 1] for c in cs]) for l in range(L)]
    vis_start = torch.tensor(bt.vis_start, dtype=torch.int32, device=DEV)
    vis_len = torch.tensor(bt.n_vis, dtype=torch.int32, device=DEV)
    # static inputs of the graph; host-side bounds are those of the last step
    seq_len_g = torch.tensor(bt.seq_len(1), dtype=torch.int32, device=DEV)
    batch_g = fo.SeqBatch(seq_len_g, vis_start, vis_len, max_seq, max_vis)
    qs_g = [q.clone() for q in queries(1)]
    outs_g = [torch.zeros_like(q) for q in qs_g]

    def eager_step(t):
        batch = fo.SeqBatch.from_lists(bt.seq_len(t), bt.vis_start, bt.n_vis, DEV)
        batch.max_seq_len = max_seq
        outs = [torch.zeros_like(q) for q in qs_g]
        eager.step(t, batch, queries(t), outs)
        return outs

    def load_inputs(t):
        seq_len_g.copy_(torch.tensor(bt.seq_len(t), dtype=torch.int32))
        for dst, src in zip(qs_g, queries(t)):
            dst.copy_(src)

    # steps 1, 2 eagerly on both (step 1 takes the fallback path; step 2 is the steady-state schedule)
    for t in (1, 2):
        ref = eager_step(t)
        load_inputs(t)
        graphed.step(t, batch_g, qs_g, outs_g)
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(ref, outs_g))
    # capture step 3's schedule (the same for every later step)
    load_inputs(3)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.step(3, batch_g, qs_g, outs_g)
    for t in range(3, steps + 1):
        ref = eager_step(t)
        load_inputs(t)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for l, (a, b) in enumerate(zip(ref, outs_g)):
            assert torch.equal(a, b), f"step {t} layer {l}: replay differs from the eager step"
        assert torch.equal(eager.kept_idx, graphed.kept_idx) and torch.equal(eager.kept_cnt, graphed.kept_cnt)
