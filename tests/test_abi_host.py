"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes workspaces, computes ceil(tau N) like the oracle, and rejects bad
arguments before any HIP call."""
import ctypes
import os
import re
from fractions import Fraction
import math

import pytest

import oracle
from paper_2605_17447_amd import binding as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000          # non-null, 256-byte aligned "device pointer"; never dereferenced on these paths


@pytest.fixture(scope="module")
def lib():
    return fb.load_library()


def _kv(dtype=fb.BF16, Hkv=4, d=128, S=4160, paged=False, **kw):
    v = fb.KvView(FAKE, FAKE, dtype, Hkv, d, d, S * d, Hkv * S * d, 0, 0, None, 0)
    if paged:
        v.page_tokens, v.stride_page, v.block_table, v.max_pages_per_seq = 64, Hkv * 64 * d, FAKE, 65
        v.stride_head = 64 * d
    for k, val in kw.items():
        setattr(v, k, val)
    return v


def _bv(B=2, S=4160, N=4096, **kw):
    v = fb.BatchView(B, FAKE, FAKE, FAKE, S, N)
    for k, val in kw.items():
        setattr(v, k, val)
    return v


def test_header_symbols_are_all_exported(lib):
    text = open(os.path.join(ROOT, "include", "fastocr.h")).read()
    declared = sorted(set(re.findall(r"\b(fastocr_[a-z_]+)\s*\(", text)))
    assert set(declared) == set(fb.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_strerror(lib):
    assert "gfx950" in fb.version()
    assert fb.strerror(0) == "ok" and "workspace" in fb.strerror(fb.EWORKSPACE)
    assert fb.strerror(-99) == "unknown status"


def test_keep_count_agrees_with_oracle_and_exact_arithmetic():
    for tau in ("0.004", "0.02", "0.05", "0.07", "0.10", "0.25", "0.55", "1.0"):
        for n in list(range(0, 600)) + [4096, 9216, 16383, 16384, 20000]:
            k = fb.keep_count(n, float(tau))
            assert k == oracle.keep_count(n, float(tau)) == math.ceil(Fraction(tau) * n)
    assert fb.keep_count(256, 0.05) == 13 and fb.keep_count(16384, 0.05) == 820
    assert fb.keep_count(100, 0.0) == 0 and fb.keep_count(100, -1.0) == 0


def test_workspace_sizes_cover_the_documented_buffers(lib):
    kv, bv = _kv(), _bv()
    Hq = 28
    w_score = lib.fastocr_workspace_bytes(fb.OP_FOCAL_SCORE, ctypes.byref(kv), ctypes.byref(bv), Hq, 0)
    # at least the parked fp32 logits [B, Hq, S]
    assert w_score >= 2 * Hq * 4160 * 4 and w_score % 256 == 0
    w_dense = lib.fastocr_workspace_bytes(fb.OP_DENSE_DECODE_ATTN, ctypes.byref(kv), ctypes.byref(bv), Hq, 0)
    w_sparse = lib.fastocr_workspace_bytes(fb.OP_SPARSE_DECODE_ATTN, ctypes.byref(kv), ctypes.byref(bv), Hq, 205)
    assert w_dense >= 2 * Hq * (128 + 2) * 4 and w_sparse >= 2 * Hq * (128 + 2) * 4
    # top-k keeps the keys in LDS; only image spans beyond its capacity park them in the workspace
    w_topk = lib.fastocr_workspace_bytes(fb.OP_TOPK_FIXATION, None, ctypes.byref(bv), 0, 205)
    assert w_topk == 0
    big = _bv(S=70000, N=65536)
    w_big = lib.fastocr_workspace_bytes(fb.OP_TOPK_FIXATION, None, ctypes.byref(big), 0, 1)
    assert w_big >= 2 * 65536 * 4 and w_big % 256 == 0
    # invalid shapes give 0
    assert lib.fastocr_workspace_bytes(fb.OP_FOCAL_SCORE, ctypes.byref(kv), ctypes.byref(bv), 30, 0) == 0
    assert lib.fastocr_workspace_bytes(99, ctypes.byref(kv), ctypes.byref(bv), Hq, 0) == 0


def _score(lib, kv, bv, Hq=28, q=FAKE, scale=0.088, scores=FAKE, ws=FAKE, ws_bytes=1 << 40):
    return lib.fastocr_focal_score(ctypes.byref(kv) if kv else None, ctypes.byref(bv) if bv else None, q, Hq,
                                   scale, scores, None, None, ws, ws_bytes, None)


def _dense(lib, kv, bv, Hq=28, q=FAKE, out=FAKE, ws=FAKE, ws_bytes=1 << 40, scale=0.088):
    return lib.fastocr_dense_decode_attn(ctypes.byref(kv), ctypes.byref(bv), q, Hq, scale, out, None, ws,
                                         ws_bytes, None)


def _focal_layer(lib, kv, bv, Hq=28, q=FAKE, out=FAKE, scores=FAKE, ws=FAKE, ws_bytes=1 << 40, scale=0.088):
    return lib.fastocr_focal_attn_score(ctypes.byref(kv) if kv else None, ctypes.byref(bv) if bv else None, q, Hq,
                                        scale, out, scores, None, None, ws, ws_bytes, None)


def test_focal_layer_call_validation_and_workspace(lib):
    kv, bv = _kv(), _bv()
    assert _focal_layer(lib, None, bv) == fb.EINVAL
    assert _focal_layer(lib, kv, bv, out=None) == fb.EINVAL
    assert _focal_layer(lib, kv, bv, scores=None) == fb.EINVAL
    assert _focal_layer(lib, kv, bv, q=FAKE + 2) == fb.EINVAL
    assert _focal_layer(lib, kv, bv, Hq=30) == fb.EINVAL
    assert _focal_layer(lib, kv, bv, scale=float("inf")) == fb.EINVAL
    assert _focal_layer(lib, _kv(dtype=7), bv) == fb.EUNSUPPORTED
    assert _focal_layer(lib, kv, bv, ws=None) == fb.EWORKSPACE
    assert _focal_layer(lib, kv, bv, ws_bytes=1024) == fb.EWORKSPACE
    assert _focal_layer(lib, kv, _bv(B=0)) == fb.OK
    # the call may fall back to the two separate calls in the same buffer: it covers both of theirs
    w = lambda op: lib.fastocr_workspace_bytes(op, ctypes.byref(kv), ctypes.byref(bv), 28, 0)
    assert w(fb.OP_FOCAL_ATTN_SCORE) >= max(w(fb.OP_FOCAL_SCORE), w(fb.OP_DENSE_DECODE_ATTN))
    assert w(fb.OP_FOCAL_ATTN_SCORE) % 256 == 0
    for key in (b"focal_fused", b"score_resident"):
        assert lib.fastocr_set_tuning(key, 3) == fb.EINVAL and lib.fastocr_set_tuning(key, -1) == fb.EINVAL
        assert lib.fastocr_set_tuning(key, 2) == fb.OK and lib.fastocr_set_tuning(key, 1) == fb.OK


def test_argument_validation_happens_before_any_gpu_work(lib):
    kv, bv = _kv(), _bv()
    assert _score(lib, None, bv) == fb.EINVAL
    assert _score(lib, kv, None) == fb.EINVAL
    assert _score(lib, kv, bv, q=None) == fb.EINVAL
    assert _score(lib, kv, bv, q=FAKE + 2) == fb.EINVAL                      # q not 16-byte aligned
    assert _score(lib, kv, bv, scale=float("nan")) == fb.EINVAL
    assert _score(lib, kv, bv, Hq=30) == fb.EINVAL                           # Hq % Hkv != 0
    assert _score(lib, kv, bv, scores=None) == fb.EINVAL
    assert _score(lib, _kv(dtype=7), bv) == fb.EUNSUPPORTED
    assert _score(lib, _kv(d=512, stride_token=512), bv) == fb.EUNSUPPORTED
    assert _score(lib, _kv(k=None), bv) == fb.EINVAL
    assert _score(lib, kv, _bv(max_vis_len=5000)) == fb.EINVAL               # span longer than the sequence
    assert _score(lib, kv, _bv(seq_len=None)) == fb.EINVAL
    assert _score(lib, kv, _bv(B=-1)) == fb.EINVAL
    assert _score(lib, _kv(stride_token=64), bv) == fb.EINVAL                # rows overlap
    # paged view whose block table is too short for max_seq_len, or missing
    assert _score(lib, _kv(paged=True, max_pages_per_seq=10), bv) == fb.EINVAL
    assert _score(lib, _kv(paged=True, block_table=None), bv) == fb.EINVAL
    # workspace
    assert _score(lib, kv, bv, ws=None) == fb.EWORKSPACE
    assert _score(lib, kv, bv, ws=FAKE + 16) == fb.EWORKSPACE
    assert _score(lib, kv, bv, ws_bytes=1024) == fb.EWORKSPACE
    assert _dense(lib, kv, bv, out=None) == fb.EINVAL
    assert _dense(lib, kv, bv, ws_bytes=16) == fb.EWORKSPACE
    # an empty batch is a valid no-op and launches nothing
    assert _score(lib, kv, _bv(B=0)) == fb.OK
    assert _dense(lib, kv, _bv(B=0)) == fb.OK


def test_topk_and_sparse_validation(lib):
    bv = _bv()
    call = lambda tau=0.05, prev_idx=None, prev_cnt=None, sel=FAKE, cnt=FAKE, kmax=205, b=bv: \
        lib.fastocr_topk_fixation(FAKE, ctypes.byref(b), tau, prev_idx, prev_cnt, sel, cnt, kmax, None, 0, None)
    assert call(tau=1.5) == fb.EINVAL and call(tau=-0.1) == fb.EINVAL and call(tau=float("nan")) == fb.EINVAL
    assert call(kmax=204) == fb.EINVAL                                        # row pitch below ceil(tau N)
    assert call(prev_idx=FAKE) == fb.EINVAL                                   # prev_idx without prev_cnt
    assert call(sel=None) == fb.EINVAL and call(cnt=None) == fb.EINVAL
    assert call(b=_bv(B=0)) == fb.OK
    big = _bv(S=70000, N=65536)
    assert call(b=big, kmax=4000) == fb.EWORKSPACE                            # needs a key buffer past the LDS cap
    kv = _kv()
    sp = lambda sel=FAKE, cnt=FAKE, kmax=205, ws_bytes=1 << 40: lib.fastocr_sparse_decode_attn(
        ctypes.byref(kv), ctypes.byref(bv), FAKE, 28, 0.088, sel, cnt, kmax, FAKE, FAKE, ws_bytes, None)
    assert sp(sel=None) == fb.EINVAL and sp(cnt=None) == fb.EINVAL and sp(kmax=0) == fb.EINVAL
    assert sp(ws_bytes=64) == fb.EWORKSPACE


def test_one_call_score_and_topk_validation_and_workspace(lib):
    kv, bv = _kv(), _bv()
    one = lambda tau=0.05, prev_idx=None, prev_cnt=None, sel=FAKE, cnt=FAKE, kmax=205, scores=FAKE, ws=FAKE, ws_bytes=1 << 40, \
        k=kv, b=bv, Hq=28: lib.fastocr_focal_score_topk(ctypes.byref(k) if k else None, ctypes.byref(b), FAKE, Hq, 0.088, tau,
                                                         prev_idx, prev_cnt, sel, cnt, kmax, scores, None, None, ws, ws_bytes, None)
    layer = lambda out=FAKE, tau=0.05, kmax=205, ws_bytes=1 << 40, b=bv: lib.fastocr_focal_attn_score_topk(
        ctypes.byref(kv), ctypes.byref(b), FAKE, 28, 0.088, tau, None, None, FAKE, FAKE, kmax, out, FAKE, None, None, FAKE, ws_bytes, None)
    assert one(tau=1.5) == fb.EINVAL and one(kmax=204) == fb.EINVAL and one(prev_idx=FAKE) == fb.EINVAL
    assert one(sel=None) == fb.EINVAL and one(scores=None) == fb.EINVAL and one(k=None) == fb.EINVAL
    assert one(Hq=30) == fb.EINVAL
    assert one(ws=None) == fb.EWORKSPACE and one(ws_bytes=1024) == fb.EWORKSPACE
    assert one(b=_bv(B=0)) == fb.OK
    assert layer(out=None) == fb.EINVAL and layer(tau=-1.0) == fb.EINVAL and layer(ws_bytes=64) == fb.EWORKSPACE
    assert layer(b=_bv(B=0)) == fb.OK
    w = lambda op, kmax=205: lib.fastocr_workspace_bytes(op, ctypes.byref(kv), ctypes.byref(bv), 28, kmax)
    assert w(fb.OP_FOCAL_SCORE_TOPK) >= max(w(fb.OP_FOCAL_SCORE), w(fb.OP_TOPK_FIXATION))
    assert w(fb.OP_FOCAL_ATTN_SCORE_TOPK) >= max(w(fb.OP_FOCAL_ATTN_SCORE), w(fb.OP_TOPK_FIXATION))
    assert lib.fastocr_workspace_bytes(fb.OP_FOCAL_SCORE_TOPK, ctypes.byref(kv), ctypes.byref(bv), 30, 205) == 0
    assert lib.fastocr_set_tuning(b"select_fused", 2) == fb.EINVAL
    assert lib.fastocr_set_tuning(b"select_fused", 1) == fb.OK and lib.fastocr_set_tuning(b"select_fused", 0) == fb.OK


def test_static_scratch_entry_point_validation(lib):
    """The entry point that allocates nothing refuses bad arguments and shapes beyond its buffer before
    any GPU call (FASTOCR_ETOOLARGE names the limit)."""
    kv, bv = _kv(), _bv()
    call = lambda k=kv, b=bv, out=FAKE, Hq=28: lib.fastocr_dense_decode_attn_static(ctypes.byref(k), ctypes.byref(b), FAKE, Hq,
                                                                                    0.088, out, None, None)
    assert call(out=None) == fb.EINVAL and call(Hq=30) == fb.EINVAL and call(k=_kv(dtype=7)) == fb.EUNSUPPORTED
    assert call(b=_bv(B=0)) == fb.OK
    big = _bv(B=4000)
    assert lib.fastocr_workspace_bytes(fb.OP_DENSE_DECODE_ATTN, ctypes.byref(kv), ctypes.byref(big), 28, 0) > fb.STATIC_SCRATCH_BYTES
    assert call(b=big) == fb.ETOOLARGE
    assert "static" in fb.strerror(fb.ETOOLARGE)


def test_stream_release_is_a_host_side_no_op_for_unknown_streams(lib):
    assert lib.fastocr_stream_release(None) == fb.OK
    assert lib.fastocr_stream_release(0x1234500) == fb.OK


def test_exchange_timeouts_rejects_a_null_pointer(lib):
    lib.fastocr_exchange_timeouts.restype = ctypes.c_int
    lib.fastocr_exchange_timeouts.argtypes = [ctypes.c_void_p]
    assert lib.fastocr_exchange_timeouts(None) == -1          # FASTOCR_EINVAL, before any GPU call


def test_pruned_attention_workspace_grows_with_the_kept_count_and_ignores_graph_replay(lib):
    """A workspace sized with a larger kmax (or none) must cover every call with a smaller one, whichever
    way the list is cut: the size is monotone in kmax and the same with "graph_replay" 0 and 1."""
    for B, Hkv, Hq, S, N in [(1, 4, 28, 4700, 4096), (4, 2, 16, 10300, 8100), (12, 2, 12, 4700, 3969), (8, 4, 28, 4400, 4096),
                             (20, 2, 16, 9000, 8100), (16, 8, 64, 17200, 16384), (40, 1, 8, 3000, 2500)]:
        kv, bv = _kv(Hkv=Hkv, S=S), _bv(B=B, S=S, N=N)
        sizes = []
        for kmax in [1, 13, 64, 205, 410, 820, 2048, N, 0]:          # 0 = unknown: the whole sequence
            w0 = lib.fastocr_workspace_bytes(fb.OP_SPARSE_DECODE_ATTN, ctypes.byref(kv), ctypes.byref(bv), Hq, kmax)
            assert lib.fastocr_set_tuning(b"graph_replay", 1) == fb.OK
            w1 = lib.fastocr_workspace_bytes(fb.OP_SPARSE_DECODE_ATTN, ctypes.byref(kv), ctypes.byref(bv), Hq, kmax)
            assert lib.fastocr_set_tuning(b"graph_replay", 0) == fb.OK
            assert w0 == w1 and w0 > 0 and w0 % 256 == 0
            sizes.append(w0)
        assert sizes == sorted(sizes), (B, Hkv, sizes)


def test_tuning_keys(lib):
    assert lib.fastocr_set_tuning(b"splits_dense", 3) == fb.OK
    kv, bv = _kv(), _bv()
    w3 = lib.fastocr_workspace_bytes(fb.OP_DENSE_DECODE_ATTN, ctypes.byref(kv), ctypes.byref(bv), 28, 0)
    assert lib.fastocr_set_tuning(b"splits_dense", 6) == fb.OK
    w6 = lib.fastocr_workspace_bytes(fb.OP_DENSE_DECODE_ATTN, ctypes.byref(kv), ctypes.byref(bv), 28, 0)
    assert w6 > w3
    assert lib.fastocr_set_tuning(b"splits_dense", 0) == fb.OK
    assert lib.fastocr_set_tuning(b"no_such_key", 1) == fb.EINVAL
    assert lib.fastocr_set_tuning(None, 1) == fb.EINVAL
    assert lib.fastocr_kernel_timer_enable(99, 4) == fb.EINVAL
    assert lib.fastocr_kernel_timer_read(0, None, 0) == 0
    assert lib.fastocr_set_tuning(b"timer_every", 0) == fb.EINVAL
    assert lib.fastocr_set_tuning(b"timer_every", 4) == fb.OK
    assert lib.fastocr_set_tuning(b"timer_every", 1) == fb.OK
    assert lib.fastocr_set_tuning(b"attn_waves", 5) == fb.EINVAL and lib.fastocr_set_tuning(b"attn_waves", 0) == fb.EINVAL
    assert lib.fastocr_set_tuning(b"attn_waves", 8) == fb.OK and lib.fastocr_set_tuning(b"attn_waves", 4) == fb.OK
    assert lib.fastocr_set_tuning(b"graph_replay", 2) == fb.EINVAL
    assert lib.fastocr_set_tuning(b"graph_replay", 1) == fb.OK and lib.fastocr_set_tuning(b"graph_replay", 0) == fb.OK
    assert lib.fastocr_set_tuning(b"exchange_fallback", 2) == fb.EINVAL
    assert lib.fastocr_set_tuning(b"exchange_fallback", 1) == fb.OK and lib.fastocr_set_tuning(b"exchange_fallback", 0) == fb.OK


def test_binding_views_follow_their_tensors():
    """The binding keeps the C views of a cache and a batch; a changed tensor, shape or maximum must
    give a new view, an unchanged one the same view."""
    import torch
    import paper_2605_17447_amd as fo
    k = torch.zeros(2, 4, 40, 128, dtype=torch.bfloat16)
    v = torch.zeros_like(k)
    cache = fo.KvCache(k, v)
    a = cache.view()
    assert cache.view() is a
    assert (a.k, a.v, a.n_kv_heads, a.head_dim, a.stride_token, a.stride_head, a.stride_seq) == \
           (k.data_ptr(), v.data_ptr(), 4, 128, 128, 40 * 128, 4 * 40 * 128)
    cache.k, cache.v = k[:, :2], v[:, :2]                     # same addresses, fewer heads
    b = cache.view()
    assert b is not a and b.n_kv_heads == 2 and b.stride_seq == 4 * 40 * 128
    k2 = torch.zeros_like(k)
    cache.k, cache.v = k2, v
    assert cache.view().k == k2.data_ptr()
    cache = fo.KvCache(k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous(), layout="bshd")
    c = cache.view()
    assert (c.stride_token, c.stride_head) == (4 * 128, 128)
    table = torch.zeros(2, 3, dtype=torch.int32)
    paged = fo.KvCache(torch.zeros(6, 4, 16, 128), torch.zeros(6, 4, 16, 128), block_table=table)
    p = paged.view()
    assert (p.page_tokens, p.stride_page, p.max_pages_per_seq, p.block_table) == (16, 4 * 16 * 128, 3, table.data_ptr())
    paged.block_table = torch.zeros(2, 5, dtype=torch.int32)
    assert paged.view().max_pages_per_seq == 5

    batch = fo.SeqBatch.from_lists([30, 40], [2, 3], [20, 25], "cpu")
    x = batch.view()
    assert batch.view() is x and (x.batch, x.max_seq_len, x.max_vis_len) == (2, 40, 25)
    batch.max_seq_len = 41
    y = batch.view()
    assert y is not x and y.max_seq_len == 41
    batch.seq_len = torch.tensor([31, 41], dtype=torch.int32)
    assert batch.view().seq_len == batch.seq_len.data_ptr()
