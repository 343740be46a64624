"""The single-launch forms (register-resident scoring, the fused focal layer, pruned attention
merged inside the launch) hand data between workgroups through static device memory, one exchange
slot per call in flight.  A slot belongs to a stream, and a captured call's slot to its graph: a
HIP-graph replay on one stream next to eager calls on another must never meet in a slot, however
many eager calls go by.  Every result is compared bit for bit with the same call run alone (the
kernels are deterministic) and against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_17447_amd as fo
from paper_2605_17447_amd import binding as fb
from util import TinyCase

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DEV, check_out, check_scores, problem_from_case


class _Run:
    """One problem's buffers and the three single-launch calls (+ top-k) on a given stream."""

    def __init__(self, case, tau):
        p = problem_from_case(case)
        self.p, self.tau = p, tau
        self.kmax = max(1, fo.keep_count(p.batch.max_vis_len, tau))
        need = max(fo.workspace_bytes(op, p.cache, p.batch, p.Hq, self.kmax) for op in range(5))
        self.ws = torch.empty(need, dtype=torch.uint8, device=DEV)
        self.sc = torch.zeros((p.B, p.batch.max_vis_len), dtype=torch.float32, device=DEV)
        self.sc2 = torch.zeros_like(self.sc)
        self.idx = torch.zeros((p.B, self.kmax), dtype=torch.int32, device=DEV)
        self.cnt = torch.zeros((p.B,), dtype=torch.int32, device=DEV)
        self.out_s, self.out_f = torch.zeros_like(p.q), torch.zeros_like(p.q)

    def enqueue(self, stream=None):
        p = self.p
        fo.focal_score(p.cache, p.batch, p.q, p.scale, self.sc, self.ws, stream=stream)
        fo.topk_fixation(self.sc, p.batch, self.tau, self.idx, self.cnt, self.ws, stream=stream)
        fo.sparse_decode_attn(p.cache, p.batch, p.q, p.scale, self.idx, self.cnt, self.out_s, self.ws, stream=stream)
        fo.focal_attn_score(p.cache, p.batch, p.q, p.scale, self.out_f, self.sc2, self.ws, stream=stream)

    def results(self):
        return [t.clone() for t in (self.sc, self.idx, self.cnt, self.out_s, self.out_f, self.sc2)]

    def clear(self):
        for t in (self.sc, self.sc2, self.idx, self.cnt, self.out_s, self.out_f):
            t.zero_()

    def check_against_oracle(self, what):
        p = self.p
        oc = p.oracle_args()
        ref_sc, _, _ = oracle.focal_score(*oc)
        check_scores(self.sc, ref_sc, p.vis_len, what + " scores")
        check_scores(self.sc2, ref_sc, p.vis_len, what + " focal-layer scores")
        idx_h, cnt_h, sc_h = self.idx.cpu().numpy(), self.cnt.cpu().numpy(), self.sc.cpu().numpy()
        for b in range(p.B):
            assert np.array_equal(idx_h[b, : cnt_h[b]], oracle.topk(sc_h[b, : p.vis_len[b]], int(cnt_h[b])))
        ref_s, _ = oracle.decode_attn(*oc, idx_h, cnt_h)
        check_out(self.out_s, ref_s, what + " pruned attention")
        check_out(self.out_f, oracle.decode_attn(*oc)[0], what + " focal-layer output")


def test_graph_replays_on_one_stream_next_to_eager_calls_on_another():
    a = _Run(TinyCase(seed=601, B=3, Hq=28, Hkv=4, d=128, n_vis=[1200, 900, 1500], pre=[10, 3, 0], post=[50, 30, 9],
                      dtype="bf16"), 0.1)
    b = _Run(TinyCase(seed=602, B=2, Hq=64, Hkv=8, d=128, n_vis=[1100, 1300], pre=[5, 0], post=[70, 20], dtype="bf16"), 0.1)
    timeouts_before = fb.exchange_timeouts()
    fb.set_tuning("splits_sparse", 3)                 # several ranges per stream: merged inside the launch
    fb.set_tuning("score_resident", 2)
    fb.set_tuning("focal_fused", 2)
    try:
        # each problem alone: the reference bits
        a.enqueue(); torch.cuda.synchronize(); want_a = a.results(); a.check_against_oracle("problem A alone")
        b.enqueue(); torch.cuda.synchronize(); want_b = b.results(); b.check_against_oracle("problem B alone")
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=sa):
            a.enqueue()
        torch.cuda.synchronize()
        # 40 rounds: a replay on stream A, four eager rounds of the other problem on stream B meanwhile (more
        # eager calls than there are slots of any kind go by during the test)
        for rnd in range(40):
            a.clear(); b.clear()
            torch.cuda.synchronize()
            with torch.cuda.stream(sa):
                g.replay()
            for _ in range(4):
                b.enqueue(stream=sb)
            torch.cuda.synchronize()
            for got, want in zip(a.results(), want_a):
                assert torch.equal(got, want), f"round {rnd}: the replayed graph's results changed"
            for got, want in zip(b.results(), want_b):
                assert torch.equal(got, want), f"round {rnd}: the eager stream's results changed"
        assert fb.exchange_timeouts() == timeouts_before
    finally:
        fb.set_tuning("splits_sparse", 0)
        fb.set_tuning("score_resident", 1)
        fb.set_tuning("focal_fused", 1)


def test_more_streams_than_exchange_slots_fall_back_to_the_separate_kernels():
    """Streams beyond the slots of a kind get the forms built from separate kernels: same results to
    the bar, no shared state.  40 streams each run the path once, all enqueued before any is waited for."""
    runs = [_Run(TinyCase(seed=700 + i, B=2, Hq=28, Hkv=4, d=128, n_vis=[700 + 13 * i, 500], pre=[4, 1], post=[30 + i, 9],
                          dtype="bf16"), 0.1) for i in range(4)]
    fb.set_tuning("splits_sparse", 2)
    try:
        streams = [torch.cuda.Stream() for _ in range(40)]
        torch.cuda.synchronize()
        for rnd in range(10):
            for i, r in enumerate(runs):
                r.clear()
            torch.cuda.synchronize()
            for i, r in enumerate(runs):
                r.enqueue(stream=streams[4 * rnd + i])
            torch.cuda.synchronize()
            for i, r in enumerate(runs):
                r.check_against_oracle(f"round {rnd}, stream {4 * rnd + i}")
    finally:
        fb.set_tuning("splits_sparse", 0)


def test_released_streams_hand_their_slots_on():
    """40 streams in turn, each released after use: every one runs the single-launch forms (no top-level
    merge kernel is ever launched), where without the release the 5th stream on would fall back."""
    run = _Run(TinyCase(seed=790, B=2, Hq=28, Hkv=4, d=128, n_vis=[900, 700], pre=[4, 1], post=[40, 9], dtype="bf16"), 0.1)
    fb.set_tuning("splits_sparse", 2)
    try:
        run.enqueue()
        torch.cuda.synchronize()
        want = run.results()
        streams = [torch.cuda.Stream() for _ in range(40)]
        fb.kernel_timer_enable(fb.KERNEL_ATTN_COMBINE, 256)
        for st in streams:
            fb.stream_release(st)                       # whatever earlier tests left on the pool's handles
        fb.kernel_timer_read(fb.KERNEL_ATTN_COMBINE)
        launched_before = 0
        for i, st in enumerate(streams):
            run.clear()
            run.enqueue(stream=st)
            st.synchronize()
            for got, w in zip(run.results(), want):
                assert torch.equal(got, w), f"stream {i}: results changed"
            fb.stream_release(st)
        # the fused focal layer always ends with its merge of the waves' partials (one launch per call); pruned
        # attention adds one only when it could not merge inside its launch
        assert len(fb.kernel_timer_read(fb.KERNEL_ATTN_COMBINE)) == len(streams)
    finally:
        fb.kernel_timer_enable(fb.KERNEL_ATTN_COMBINE, 0)
        fb.set_tuning("splits_sparse", 0)


def test_calls_from_several_host_threads_each_on_its_own_stream():
    """The binding releases the interpreter lock inside the C calls, so threads really run the library's host
    code side by side: the slot tables, tuning values and per-device words are guarded for that."""
    import threading
    runs = [_Run(TinyCase(seed=760 + i, B=2, Hq=28, Hkv=4, d=128, n_vis=[800 + 31 * i, 600], pre=[4, 1], post=[40 + i, 9],
                          dtype="bf16"), 0.1) for i in range(4)]
    fb.set_tuning("splits_sparse", 2)
    try:
        for r in runs:
            r.enqueue()
        torch.cuda.synchronize()
        want = [r.results() for r in runs]
        errors = []

        def work(i):
            try:
                st = torch.cuda.Stream()
                for _ in range(25):
                    runs[i].enqueue(stream=st)
                    fb.set_tuning("timer_every", 1)            # a writer among the readers
                st.synchronize()
            except Exception as e:                              # surfaced in the main thread
                errors.append(e)

        threads = [threading.Thread(target=work, args=(i,)) for i in range(4)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        torch.cuda.synchronize()
        assert not errors, errors
        for i, r in enumerate(runs):
            for got, w in zip(r.results(), want[i]):
                assert torch.equal(got, w), f"thread {i}: results changed"
    finally:
        fb.set_tuning("splits_sparse", 0)
