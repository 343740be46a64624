"""Benchmark of the FastOCR decode hot path on one MI355X.

A "step" is one three-step layer-step on one attention layer for the whole batch: focal
scoring of the current queries against all cached keys, top-k of ceil(tau N) image tokens
warm-started from the previous step's set, and sparse decode attention over text + selected
image tokens.  Workload: the large dense-document configuration (bf16, batch 16, Hq 64, Hkv 8,
head_dim 128, N = 16384 image tokens, 256-token text prefix, mid-run text length), tau = 0.05,
synthetic drifting-fixation queries; the sequence grows by one token per step.  Consecutive steps
alternate between `--layers` (default 2) distinct caches of that shape, as consecutive layer-steps
of a model do, so that no step finds its K/V in the 256 MB memory-side cache from the step before.
Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line.  The dense decode-attention comparator and the per-kernel breakdown are
measured in separate passes after the timed region and reported as extra keys.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload configuration (4 = the metric's)")
    ap.add_argument("--tau", type=float, default=0.05)
    ap.add_argument("--batch", type=int, default=0, help="override the configuration's batch size")
    ap.add_argument("--start-step", type=int, default=0, help="decode step the run starts at (0 = mid-run)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--time-every", type=int, default=4,
                    help="launches of the dominant kernel between two that carry HIP events (an event pair costs the "
                         "stream about 4.5 us; 1 = every launch)")
    ap.add_argument("--no-extras", action="store_true", help="skip the comparator / breakdown passes")
    ap.add_argument("--stacks", default="3,5,4,t2a,t2c", help="stacks measured in the extras: 28-layer stacks by configuration shape "
                                                        "(3: batch 8, N 4096; 5: ragged paged batch 32, 18 GB; 4: the metric "
                                                        "workload's shape, 33 GB); empty = none")
    ap.add_argument("--cpu-budget-s", type=float, default=12.0)
    ap.add_argument("--layers", type=int, default=2, help="distinct caches the steps rotate over")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch the plain copy / read probe kernels of known size (1 GiB) three times "
                         "each, so that a profiler's byte counters can be scaled against them")
    ap.add_argument("--counter-pass", action="store_true",
                    help="inputs for hardware-counter passes: the caches are filled by one random-normal launch each "
                         "(the same distribution as the seeded generator's, which takes thousands of small launches: "
                         "under the counter collection on this pool such runs have stalled before reaching the "
                         "library's kernels) and every step uses one set of queries drawn on the host; shapes, "
                         "dtypes and launch configurations are unchanged, and the bytes a launch moves do not "
                         "depend on the values")
    ap.add_argument("--step", choices=["three_step", "focal_layer"], default="three_step",
                    help="what one timed step is: the metric's three-step path (default), or a focal layer as "
                         "the controller runs it (dense output + scores from one pass over K and V, then top-k); "
                         "the roofline object then describes the fused kernel")
    ap.add_argument("--paged", action="store_true",
                    help="keep the configuration's paged KV layout (configuration 5) instead of a contiguous cache")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="launch-shape override passed to fastocr_set_tuning (measurement sweeps)")
    return ap.parse_args()


def kernel_sources_sha256(names):
    """Digest of the source files a kernel is built from (the profile summaries under profiles/ record the
    digest they were taken with, so that a stale traffic figure is not reported for a changed kernel)."""
    import hashlib
    h = hashlib.sha256()
    for n in names:
        with open(os.path.join(ROOT, "paper_2605_17447_amd", "csrc", n), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


# The settings of the paper's efficiency table (Table 2: batch, prompt length including the image tokens /
# tokens generated) as attention-only stacks.  The paper prints neither model's head shape; these are the public
# configurations of a 3B-class decoder (36 layers, 16 query / 2 KV heads, head_dim 128) and a 1.7B-class one
# (28 layers, 12 / 2 heads), with floor(0.1 L) focal layers at least two layers apart (Sec. 4.1's defaults:
# focal layer ratio 0.1, focal gap 1, kept ratio 0.05).  The image is a square grid and the text prefix fills
# the prompt up to its length.  paper_ms = (vanilla, FastOCR) attention latency per step in Table 2, measured
# by its authors on other hardware with their framework's attention: context, not a target.
TABLE2_STACKS = {
    "t2a": dict(label="3B-class decoder, batch 12, prompt 4096 / 1024 generated", paper_ms=(26.00, 8.69),
                over=dict(batch=12, n_q_heads=16, n_kv_heads=2, n_layers=36, focal_layers=(17, 19, 21), focal_gap=1,
                          n_visual=(3969, 3969), grid_w=(63, 63), text_prefix=(127, 127), steps=1024)),
    "t2b": dict(label="3B-class decoder, batch 4, prompt 8192 / 2048 generated", paper_ms=(17.70, 7.96),
                over=dict(batch=4, n_q_heads=16, n_kv_heads=2, n_layers=36, focal_layers=(17, 19, 21), focal_gap=1,
                          n_visual=(8100, 8100), grid_w=(90, 90), text_prefix=(92, 92), steps=2048)),
    "t2c": dict(label="1.7B-class decoder, batch 12, prompt 4096 / 1024 generated", paper_ms=(15.55, 5.57),
                over=dict(batch=12, n_q_heads=12, n_kv_heads=2, n_layers=28, focal_layers=(16, 20), focal_gap=1,
                          n_visual=(3969, 3969), grid_w=(63, 63), text_prefix=(127, 127), steps=1024)),
    "t2d": dict(label="1.7B-class decoder, batch 4, prompt 8192 / 2048 generated", paper_ms=(10.62, 5.51),
                over=dict(batch=4, n_q_heads=12, n_kv_heads=2, n_layers=28, focal_layers=(16, 20), focal_gap=1,
                          n_visual=(8100, 8100), grid_w=(90, 90), text_prefix=(92, 92), steps=2048)),
}


def stack_extras(fs, fo, torch, np, dev, tau, cfg, n_time=30, **over):
    """Measured (not modelled) blend of focal and pruned layers: a 28-layer attention-only stack with
    focal layers {2, 14} driven by the step controller, one decode step captured in a HIP graph and
    replayed (the sequences grow by one token per replay), against 28 dense attention layers captured
    the same way.  cfg 3: batch 8, N = 4096 (launch-bound shapes); cfg 5: batch 32, ragged image spans
    up to 16384 tokens, paged; cfg 4 with n_layers=28: the metric workload's shape as a stack.  Every
    layer has its own generated cache.  The captured FastOCR step is taken with the library's
    "graph_replay" hint set (short lists of few streams are cut finer when launches follow each other
    closely); the eager figure and the dense stack are not affected by it."""
    over = dict(over)
    t_start = over.pop("steps", fs.config(cfg).steps) // 2        # mid-run, like the single-layer measurement
    wl = fs.config(cfg, steps=t_start + n_time + 16, warmup=0, **over)
    L, focal = wl.n_layers, wl.focal_layers
    bts = [fs.make_batch(wl, device=dev, layer=l) for l in range(L)]
    bt = bts[0]
    progress("stack config %d: %d caches generated" % (cfg, L))
    cs = fs.centres(bt, t_start + 4)
    B, Hq, d = wl.batch, wl.n_q_heads, wl.head_dim
    scale = float(np.float32(d ** -0.5))
    caches = [fo.KvCache(x.k, x.v, "bhsd", x.block_table) for x in bts]
    max_seq, max_vis = max(bt.seq_len(wl.steps)), max(bt.n_vis)
    ctl = fo.FixationController(caches, Hq, scale, focal, tau, 0, max_seq, max_vis, B, dev, focal_gap=wl.focal_gap)
    seq_len = torch.tensor(bt.seq_len(t_start), dtype=torch.int32, device=dev)
    batch = fo.SeqBatch(seq_len, torch.tensor(bt.vis_start, dtype=torch.int32, device=dev),
                        torch.tensor(bt.n_vis, dtype=torch.int32, device=dev), max_seq, max_vis)
    qs = [fs.queries_for_step(bts[l], t_start + 2, [c[t_start + 1] for c in cs]) for l in range(L)]
    outs = [torch.zeros_like(q) for q in qs]
    for t in (1, 2):                                   # fallback step, then the steady-state schedule
        ctl.step(t, batch, qs, outs)
        seq_len.add_(1)
    torch.cuda.synchronize()

    def timed(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / n

    eager_us = timed(lambda: (ctl.step(3, batch, qs, outs), seq_len.add_(1)), 5)
    ctl.graph_replay = True                            # the captured step is told that it will be replayed
    try:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            ctl.step(3, batch, qs, outs)
    finally:
        ctl.graph_replay = False
    timed(lambda: (g.replay(), seq_len.add_(1)), 3)
    graph_us = timed(lambda: (g.replay(), seq_len.add_(1)), n_time)
    seq_len.copy_(torch.tensor(bt.seq_len(t_start + 2), dtype=torch.int32))
    ws = torch.empty(max(fo.workspace_bytes(3, c, batch, Hq, 0) for c in caches[:1]), dtype=torch.uint8, device=dev)
    dense = lambda: [fo.dense_decode_attn(caches[l], batch, qs[l], scale, outs[l], ws) for l in range(L)]
    dense()
    torch.cuda.synchronize()
    gd = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gd):
        dense()
    timed(lambda: (gd.replay(), seq_len.add_(1)), 3)
    dense_us = timed(lambda: (gd.replay(), seq_len.add_(1)), n_time)
    e = 2 if wl.dtype == "bf16" else 4
    R = wl.n_kv_heads * d * e
    kv_gb = sum(x.k.numel() + x.v.numel() for x in bts) * e / 1e9
    # bytes the method must move per decode step: focal layers read all of K and V once, the others text + kept rows
    s_mid = [n + bt.prefix[b] + t_start + 2 + (11 + n_time) // 2 for b, n in enumerate(bt.n_vis)]
    dense_b = sum(s * 2 * R for s in s_mid)
    sparse_b = sum((fo.keep_count(n, tau) + s - n) * 2 * R for s, n in zip(s_mid, bt.n_vis))
    step_bytes = len(focal) * dense_b + (L - len(focal)) * sparse_b
    progress("stack config %d measured" % cfg)
    return {"workload": "config%d shape %s: %d attention layers (%.1f GB of K and V, a generated cache per layer), batch %d, Hq %d, "
                        "Hkv %d, N %s, %s, focal layers %s, tau %g, decode steps from %d on (mid-run text length), one decode step per HIP-graph replay"
                        % (cfg, wl.name, L, kv_gb, B, Hq, wl.n_kv_heads,
                           max_vis if min(bt.n_vis) == max_vis else "%d..%d" % (min(bt.n_vis), max_vis),
                           "paged" if wl.paged else "contiguous", list(focal), tau, t_start + 2),
            "fastocr_step_us": round(graph_us, 1), "dense_step_us": round(dense_us, 1),
            "measured_speedup_vs_dense": round(dense_us / graph_us, 3),
            "fastocr_step_us_without_graph": round(eager_us, 1),
            "fastocr_step_algorithmic_GBs": round(step_bytes / graph_us / 1e3, 1),
            "fastocr_step_frac_of_peak": round(step_bytes / graph_us / 1e3 / HBM_PEAK_GBS, 4),
            "dense_step_GBs": round(L * dense_b / dense_us / 1e3, 1)}


def progress(msg):
    """Stage markers on stderr when FASTOCR_BENCH_PROGRESS is set (long profiler runs)."""
    if os.environ.get("FASTOCR_BENCH_PROGRESS"):
        print("[bench] " + msg, file=sys.stderr, flush=True)


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (sequences are independent; "
              "a data-parallel job is N copies of this run). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import fastocr_synth as fs
    import paper_2605_17447_amd as fo
    from paper_2605_17447_amd import binding as fb

    progress("torch imported")
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    fo.load_library()
    for kv_ in args.tune:
        key, val = kv_.split("=")
        fb.set_tuning(key, int(val))

    n_steps, n_warm = args.steps, args.warmup
    total = n_steps + n_warm
    over = {"batch": args.batch} if args.batch else {}
    if not args.paged:
        over["paged"] = False
    wl = fs.config(args.config, n_layers=1, focal_layers=(0,), **over)
    t_first = args.start_step or max(1, wl.steps // 2 - total // 2)
    assert t_first + total - 1 <= wl.steps, "not enough decode steps in this configuration"
    tau = args.tau

    # ---- inputs (resident before timing) ---------------------------------------------------
    L = max(1, args.layers)
    bts = [fs.make_batch(wl, device=dev, layer=l, plain_fill=args.counter_pass) for l in range(L)]
    bt = bts[0]
    progress("caches generated")
    cs = fs.centres(bt, t_first + total)
    progress("fixation centres generated")
    B, Hq, Hkv, d = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    if args.counter_pass:
        # drawn on the host and copied: no generator launch runs under the counter collection
        gen = torch.Generator().manual_seed(fs.BASE_SEED)
        q1 = torch.randn((B, Hq, d), generator=gen, dtype=torch.float32).to(wl.torch_dtype).to(dev)
        qs = q1.unsqueeze(0).expand(total, B, Hq, d)
    else:
        qs = torch.stack([fs.queries_for_step(bts[i % L], t_first + i, [c[t_first + i - 1] for c in cs])
                          for i in range(total)])
    progress("queries generated")
    seq_lens = torch.tensor([bt.seq_len(t_first + i) for i in range(total)], dtype=torch.int32, device=dev)
    vis_start = torch.tensor(bt.vis_start, dtype=torch.int32, device=dev)
    vis_len = torch.tensor(bt.n_vis, dtype=torch.int32, device=dev)
    max_vis = max(bt.n_vis)
    batches = [fo.SeqBatch(seq_lens[i], vis_start, vis_len, max(bt.seq_len(t_first + i)), max_vis) for i in range(total)]
    layer_caches = [fo.KvCache(x.k, x.v, "bhsd", x.block_table) if wl.paged else fo.KvCache(x.k, x.v) for x in bts]
    caches = [layer_caches[i % L] for i in range(total)]
    cache = layer_caches[0]
    scale = float(np.float32(d ** -0.5))
    kmax = max(1, fo.keep_count(max_vis, tau))
    need = max(fo.workspace_bytes(op, cache, batches[-1], Hq, kmax) for op in range(7))
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    scores = torch.zeros((B, max_vis), dtype=torch.float32, device=dev)
    idx = torch.zeros((B, kmax), dtype=torch.int32, device=dev)
    cnt = torch.zeros((B,), dtype=torch.int32, device=dev)
    out = torch.zeros((B, Hq, d), dtype=wl.torch_dtype, device=dev)
    out_dense = torch.zeros_like(out)
    state = {"have_prev": False}

    def three_step(i):
        # scoring and the top-k through the one-call entry point (two launches: the select inside the scoring
        # launch is measured slower and is not the library's default), then pruned attention
        cache = caches[i]
        warm = state["have_prev"]
        fo.focal_score_topk(cache, batches[i], qs[i], scale, tau, scores, idx, cnt, ws,
                            prev_idx=idx if warm else None, prev_cnt=cnt if warm else None)
        state["have_prev"] = True
        fo.sparse_decode_attn(cache, batches[i], qs[i], scale, idx, cnt, out, ws)

    def focal_layer_step(i):
        warm = state["have_prev"]
        fo.focal_attn_score_topk(caches[i], batches[i], qs[i], scale, tau, out_dense, scores, idx, cnt, ws,
                                 prev_idx=idx if warm else None, prev_cnt=cnt if warm else None)
        state["have_prev"] = True

    focal_mode = args.step == "focal_layer"
    step_fn = focal_layer_step if focal_mode else three_step
    timed_kernel = fb.KERNEL_FOCAL_FUSED if focal_mode else fb.KERNEL_SCORE_LOGITS

    progress("inputs resident")
    # ---- timed region ------------------------------------------------------------------------
    # The kernel timer is set up before the warm-up steps (its events are created there), so that the GPU
    # does not sit idle between the warm-up and the timed steps for longer than the synchronize takes.
    every = max(1, args.time_every)
    fb.set_tuning("timer_every", every)
    fb.kernel_timer_enable(timed_kernel, (total + every - 1) // every + 1)
    for i in range(n_warm):
        step_fn(i)
    torch.cuda.synchronize()
    fb.kernel_timer_read(timed_kernel)          # drops the warm-up steps' samples
    t0 = time.perf_counter()
    for i in range(n_warm, total):
        step_fn(i)
    issued = time.perf_counter() - t0           # host time to issue every launch (the GPU must be the slower side)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    progress("timed region done")
    logits_ms = fb.kernel_timer_read(timed_kernel)
    fb.kernel_timer_enable(timed_kernel, 0)
    fb.set_tuning("timer_every", 1)

    if args.calibrate:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        for _ in range(3):
            fb.stream_probe(src, dst, sink)          # reads 1 GiB, writes 1 GiB
        for _ in range(3):
            fb.stream_probe(src, None, sink)         # reads 1 GiB
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = elapsed * 1e3 / n_steps
    value = n_steps / elapsed

    # ---- roofline of the dominant kernel (the K stream of focal scoring) ---------------------
    e = 2 if wl.dtype == "bf16" else 4
    R = Hkv * d * e
    mean_S = float(seq_lens[n_warm:].float().mean().item())
    scores_out = 4 * float(sum(bt.n_vis))                       # the fp32 scores written
    score_bytes = B * (mean_S * R + Hq * d * e) + scores_out    # K rows of every cached token + the queries + the scores
    if focal_mode:
        score_bytes = B * (mean_S * 2 * R + 2 * Hq * d * e) + scores_out     # K and V rows, queries in, outputs and scores out
    k_ms = float(np.mean(logits_ms)) if logits_ms else float("nan")
    achieved = score_bytes / (k_ms * 1e-3) / 1e9
    traffic, traffic_source = None, None
    prof = os.path.join(ROOT, "profiles", "focal_layer_config4_tau0.05.md" if focal_mode else "three_step_config4_tau0.05.md")
    kernel_files = (["focal_fused.hip"] if focal_mode else ["score_resident.hip"]) + ["resident.hpp", "common.hpp", "kernels.hpp"]
    if wl.config_id == 4 and abs(tau - 0.05) < 1e-12 and not args.batch and os.path.exists(prof):
        # HBM bytes per launch of this kernel from the committed rocprofv3 --pmc summary of this command; only
        # reported while the kernel's sources are the ones the summary was taken with
        for line in open(prof):
            if line.startswith("machine-readable:"):
                rec = json.loads(line.split(":", 1)[1])
                same = rec.get("kernel_sources_sha256") == kernel_sources_sha256(kernel_files)
                traffic = rec["traffic_bytes_per_launch"] if same else None
                traffic_source = {"file": os.path.relpath(prof, ROOT), "kernel_sources_sha256": rec.get("kernel_sources_sha256"),
                                  "kernel_sources_unchanged": same}
    # the whole path against the same peak: the bytes the three steps must move per step (K once, the kept
    # K and V rows, scores out and in, sets, queries, outputs) over the step time
    keep = [fo.keep_count(n, tau) for n in bt.n_vis]
    tn = [float(seq_lens[n_warm:, b].float().mean().item()) - n for b, n in enumerate(bt.n_vis)]
    path_bytes = sum((n + t_) * R + (k_ + t_) * 2 * R + 8 * n + 12 * k_ + 3 * Hq * d * e for n, t_, k_ in zip(bt.n_vis, tn, keep))
    if focal_mode:
        path_bytes = sum((n + t_) * 2 * R + 8 * n + 8 * k_ + 2 * Hq * d * e for n, t_, k_ in zip(bt.n_vis, tn, keep))
    path_gbs = path_bytes / (ms_per_step * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "focal_fused_kernel (focal layer: K and V stream, dense output and scores)" if focal_mode
                else "score_resident_kernel (focal scoring: K stream, softmax weights kept in registers)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_source,
                "path_frac": round(path_gbs / HBM_PEAK_GBS, 4), "path_achieved": round(path_gbs, 1),
                "path_algorithmic_bytes": int(path_bytes),
                "algorithmic_bytes": int(score_bytes), "avg_launch_us": round(k_ms * 1e3, 2),
                "launch_us_p10_p50_p90": [round(float(np.percentile(logits_ms, p)) * 1e3, 2) for p in (10, 50, 90)]
                if logits_ms else None,
                "launches": len(logits_ms), "timed_every": every}

    result = {
        "metric": ("decode attn layer-steps/s (focal layer: dense attention + focal score in one pass, + top-k) at N=%d, tau=%g"
                   if focal_mode else
                   "decode attn layer-steps/s (focal score + top-k + sparse attention) at N=%d, tau=%g") % (max_vis, tau),
        "value": round(value, 2), "unit": "layer-steps/s", "n_gpus": 1, "steps": n_steps, "warmup": n_warm,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": "config%d %s: batch %d, Hq %d, Hkv %d, head_dim %d, N %d visual + %d-token text "
                               "prefix, decode steps %d..%d, tau %g, warm-started top-k, steps rotate "
                               "over %d distinct caches"
                               % (wl.config_id, wl.name, B, Hq, Hkv, d, max_vis, bt.prefix[0], t_first + n_warm,
                                  t_first + total - 1, tau, L)
                               + (", caches filled by plain random-normal launches and one set of host-drawn queries for every step "
                                  "(counter pass)" if args.counter_pass else "")},
        "roofline": roofline,
        "sequence_layer_steps_per_s": round(value * B, 1),
        "host_issue_ms_per_step": round(issued * 1e3 / n_steps, 5),
    }

    # ---- extras: comparator and per-kernel breakdown (outside the timed region) ---------------
    if not args.no_extras and not focal_mode:
        names = {fb.KERNEL_SCORE_LOGITS: "score_logits", fb.KERNEL_SCORE_FINALIZE: "score_finalize",
                 fb.KERNEL_TOPK: "topk", fb.KERNEL_SPARSE_ATTN: "sparse_attn", fb.KERNEL_DENSE_ATTN: "dense_attn",
                 fb.KERNEL_ATTN_COMBINE: "attn_combine", fb.KERNEL_FOCAL_FUSED: "focal_fused"}
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_warm, total):
            fo.dense_decode_attn(caches[i], batches[i], qs[i], scale, out_dense, ws)
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - t0) * 1e3 / n_steps
        t0 = time.perf_counter()
        for i in range(n_warm, total):
            fo.sparse_decode_attn(caches[i], batches[i], qs[i], scale, idx, cnt, out, ws)
        torch.cuda.synchronize()
        sparse_ms = (time.perf_counter() - t0) * 1e3 / n_steps
        # a focal layer as the controller runs it: dense output + scores from one pass, then top-k
        for i in range(n_warm):
            fo.focal_attn_score(caches[i], batches[i], qs[i], scale, out_dense, scores, ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_warm, total):
            fo.focal_attn_score(caches[i], batches[i], qs[i], scale, out_dense, scores, ws)
            fo.topk_fixation(scores, batches[i], tau, idx, cnt, ws, prev_idx=idx, prev_cnt=cnt)
        torch.cuda.synchronize()
        focal_ms = (time.perf_counter() - t0) * 1e3 / n_steps
        for kid in names:
            fb.kernel_timer_enable(kid, 4 * n_steps)
        for i in range(n_warm, total):
            three_step(i)
            fo.dense_decode_attn(caches[i], batches[i], qs[i], scale, out_dense, ws)
            fo.focal_attn_score(caches[i], batches[i], qs[i], scale, out_dense, scores, ws)
        torch.cuda.synchronize()
        kernels_us = {}
        for kid, nm in names.items():
            ms = fb.kernel_timer_read(kid)
            kernels_us[nm] = round(float(np.mean(ms)) * 1e3, 2) if ms else None
            fb.kernel_timer_enable(kid, 0)
        dense_bytes = B * (mean_S * 2 * R + 2 * Hq * d * e)
        # what a plain read-only stream reaches on this machine (2 GiB, a trivial kernel of the library)
        probe_src = torch.empty(1 << 31, dtype=torch.uint8, device=dev).fill_(1)
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        fb.stream_probe(probe_src, None, sink)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(5):
            fb.stream_probe(probe_src, None, sink)
        ev1.record()
        torch.cuda.synchronize()
        read_ceiling = 5 * float(1 << 31) / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
        del probe_src
        # per sequence: its own kept count and its own text length (ragged batches differ in both)
        sparse_bytes = sum((fo.keep_count(n, tau) + float(seq_lens[n_warm:, b].float().mean().item()) - n) * 2 * R
                           + 4 * fo.keep_count(n, tau) + 2 * Hq * d * e for b, n in enumerate(bt.n_vis))
        focal_separate_ms = ms_per_step - sparse_ms + dense_ms   # dense output, scores and top-k as three calls
        blend = lambda f: f * focal_ms + (1 - f) * sparse_ms
        result["extras"] = {
            "dense_ms_per_layer_step": round(dense_ms, 5),
            "sparse_ms_per_layer_step": round(sparse_ms, 5),
            "focal_layer_ms_per_layer_step": round(focal_ms, 5),
            "focal_layer_ms_as_separate_calls": round(focal_separate_ms, 5),
            "focal_layer_achieved_GBs": round(dense_bytes / (focal_ms * 1e-3) / 1e9, 1),
            "dense_layer_steps_per_s": round(1e3 / dense_ms, 2),
            "speedup_three_step_vs_dense": round(dense_ms / ms_per_step, 3),
            "speedup_sparse_vs_dense": round(dense_ms / sparse_ms, 3),
            "modelled_blended_speedup_vs_dense": {"focal_fraction_0.1": round(dense_ms / blend(0.1), 3),
                                                  "focal_fraction_2_of_28": round(dense_ms / blend(2 / 28), 3),
                                                  "how": "a formula over the separately timed calls above; the measured stacks are below"},
            "measured_read_stream_ceiling_GBs": round(read_ceiling, 1),
            "dense_achieved_GBs": round(dense_bytes / (dense_ms * 1e-3) / 1e9, 1),
            "sparse_achieved_GBs": round(sparse_bytes / (sparse_ms * 1e-3) / 1e9, 1),
            "kernels_us": kernels_us,
            "paper_context": "paper reports 3.0x lower attention latency (26.00 -> 8.69 ms/step, whole model, "
                             "Qwen2.5-VL 3B, batch 12, Nvidia H800): other hardware, not a target",
        }

        # measured stacks: free this run's caches first (the largest stack holds 33 GB by itself)
        stacks = [x.strip() for x in args.stacks.split(",") if x.strip()]
        result["extras"]["measured_stacks"] = {}
        if stacks:
            keep_for_cpu = None if args.no_cpu_baseline else [(x.k.cpu(), x.v.cpu()) for x in bts]
            for x in bts:
                x.k = x.v = None
            del caches, layer_caches, cache
            torch.cuda.empty_cache()
            for name in stacks:
                if name in TABLE2_STACKS:
                    spec = TABLE2_STACKS[name]
                    r = stack_extras(fs, fo, torch, np, dev, 0.05, 3, **spec["over"])
                    r["workload"] = "Table 2 setting, " + spec["label"] + ": " + r["workload"].split(": ", 1)[1]
                    r["paper_attention_latency_ms_vanilla_fastocr"] = list(spec["paper_ms"])
                    r["paper_speedup"] = round(spec["paper_ms"][0] / spec["paper_ms"][1], 2)
                    result["extras"]["measured_stacks"]["table2_" + name[2:]] = r
                else:
                    c = int(name)
                    over = dict(n_layers=28, focal_layers=(2, 14), focal_gap=8) if c == 4 else {}
                    result["extras"]["measured_stacks"]["config%d_shape" % c] = stack_extras(fs, fo, torch, np, dev, tau, c, **over)
                torch.cuda.empty_cache()
            if keep_for_cpu is not None:
                for x, (k_, v_) in zip(bts, keep_for_cpu):
                    x.k, x.v = k_, v_

    # ---- the oracle timed on this machine's host cores (a baseline, not a target) -----------------
    if not args.no_cpu_baseline and not focal_mode:
        import oracle
        threads = oracle.max_threads()
        n_seq, cpu_s, n_steps_cpu = 0, 0.0, 0
        i = total - 1
        while cpu_s < args.cpu_budget_s:
            t_dec = t_first + i
            src = bts[i % L]
            for b in range(B):
                ok = oracle.Cache.from_bhsd(fs.to_oracle_array(src.k[b:b + 1]), fs.to_oracle_array(src.v[b:b + 1]))
                q1 = fs.to_oracle_array(qs[i][b:b + 1])
                geo = ([bt.seq_len(t_dec)[b]], [bt.vis_start[b]], [bt.n_vis[b]])
                t0 = time.perf_counter()
                sc, _, _ = oracle.focal_score(ok, *geo, q1, scale, n_threads=threads)
                sel, c = oracle.topk_fixation(sc, geo[2], tau)
                oracle.decode_attn(ok, *geo, q1, scale, sel, c, n_threads=threads)
                cpu_s += time.perf_counter() - t0
                n_seq += 1
                if cpu_s >= args.cpu_budget_s:
                    break
            n_steps_cpu += 1
            i = (i - 1) % total            # a short run's steps are taken again until the time budget is spent
        # the same oracle on one thread, one sequence-step (context for the all-core figure)
        src = bts[(total - 1) % L]
        ok1 = oracle.Cache.from_bhsd(fs.to_oracle_array(src.k[0:1]), fs.to_oracle_array(src.v[0:1]))
        q1 = fs.to_oracle_array(qs[total - 1][0:1])
        geo = ([bt.seq_len(t_first + total - 1)[0]], [bt.vis_start[0]], [bt.n_vis[0]])
        t0 = time.perf_counter()
        sc, _, _ = oracle.focal_score(ok1, *geo, q1, scale, n_threads=1)
        sel, c = oracle.topk_fixation(sc, geo[2], tau)
        oracle.decode_attn(ok1, *geo, q1, scale, sel, c, n_threads=1)
        one_thread_s = time.perf_counter() - t0
        result["cpu_baseline"] = {
            "value": round(n_seq / (B * cpu_s), 5), "unit": "layer-steps/s", "cores": threads, "kind": "oracle",
            "single_thread_value": round(1.0 / (B * one_thread_s), 5),
            "sample": "%d sequence-steps (batch %d, decode steps %d backwards, %d step(s) of the %d-step run, taken again in "
                      "turn until the %.0f s time budget was spent) of the whole three-step path, %.1f s of CPU time; "
                      "rate scaled to the full batch"
                      % (n_seq, B, t_first + total - 1, min(n_steps_cpu, total), total, args.cpu_budget_s, cpu_s)}

    print(json.dumps(result))


if __name__ == "__main__":
    main()
