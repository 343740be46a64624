"""ctypes binding of libfastocr.so: argument marshalling only.

Every step of the hot path runs in the HIP kernels behind the C ABI (include/fastocr.h);
torch is used for device memory and the stream handle, nothing else.  There is no CPU
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# FASTOCR_LIB names another build of the same library (the host-sanitized one of the CPU tests)
LIB_PATH = os.environ.get("FASTOCR_LIB") or os.path.join(_HERE, "libfastocr.so")

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP, ETOOLARGE = 0, -1, -2, -3, -4, -5
STATIC_SCRATCH_BYTES = 8 << 20
F32, BF16 = 0, 1
OP_FOCAL_SCORE, OP_TOPK_FIXATION, OP_SPARSE_DECODE_ATTN, OP_DENSE_DECODE_ATTN, OP_FOCAL_ATTN_SCORE = 0, 1, 2, 3, 4
OP_FOCAL_SCORE_TOPK, OP_FOCAL_ATTN_SCORE_TOPK = 5, 6
(KERNEL_SCORE_LOGITS, KERNEL_SCORE_FINALIZE, KERNEL_TOPK, KERNEL_SPARSE_ATTN, KERNEL_DENSE_ATTN,
 KERNEL_ATTN_COMBINE, KERNEL_FOCAL_FUSED) = range(7)

EXPORTS = (
    "fastocr_keep_count", "fastocr_workspace_bytes", "fastocr_focal_score", "fastocr_topk_fixation",
    "fastocr_sparse_decode_attn", "fastocr_dense_decode_attn", "fastocr_dense_decode_attn_static", "fastocr_focal_attn_score",
    "fastocr_focal_score_topk", "fastocr_focal_attn_score_topk", "fastocr_kernel_timer_enable",
    "fastocr_kernel_timer_read", "fastocr_select_focal_layers", "fastocr_stream_probe", "fastocr_set_tuning", "fastocr_exchange_timeouts", "fastocr_stream_release", "fastocr_strerror", "fastocr_version",
)


class KvView(ctypes.Structure):
    _fields_ = [
        ("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("dtype", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("stride_token", ctypes.c_int64), ("stride_head", ctypes.c_int64), ("stride_seq", ctypes.c_int64),
        ("page_tokens", ctypes.c_int32), ("stride_page", ctypes.c_int64),
        ("block_table", ctypes.c_void_p), ("max_pages_per_seq", ctypes.c_int32),
    ]


class BatchView(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("seq_len", ctypes.c_void_p), ("vis_start", ctypes.c_void_p),
        ("vis_len", ctypes.c_void_p), ("max_seq_len", ctypes.c_int32), ("max_vis_len", ctypes.c_int32),
    ]


class FastOcrError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} ({status})")


_lib = None


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """dlopen libfastocr.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from ._build import build
        build()
    lib = ctypes.CDLL(LIB_PATH)
    P, I, I64, F, D, SZ = (ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float,
                           ctypes.c_double, ctypes.c_size_t)
    KV, BV = ctypes.POINTER(KvView), ctypes.POINTER(BatchView)
    lib.fastocr_keep_count.restype, lib.fastocr_keep_count.argtypes = I64, [I64, D]
    lib.fastocr_workspace_bytes.restype, lib.fastocr_workspace_bytes.argtypes = SZ, [I, KV, BV, I, I64]
    lib.fastocr_focal_score.restype = I
    lib.fastocr_focal_score.argtypes = [KV, BV, P, I, F, P, P, P, P, SZ, P]
    lib.fastocr_topk_fixation.restype = I
    lib.fastocr_topk_fixation.argtypes = [P, BV, D, P, P, P, P, I64, P, SZ, P]
    lib.fastocr_sparse_decode_attn.restype = I
    lib.fastocr_sparse_decode_attn.argtypes = [KV, BV, P, I, F, P, P, I64, P, P, SZ, P]
    lib.fastocr_dense_decode_attn.restype = I
    lib.fastocr_dense_decode_attn.argtypes = [KV, BV, P, I, F, P, P, P, SZ, P]
    lib.fastocr_dense_decode_attn_static.restype = I
    lib.fastocr_dense_decode_attn_static.argtypes = [KV, BV, P, I, F, P, P, P]
    lib.fastocr_focal_attn_score.restype = I
    lib.fastocr_focal_attn_score.argtypes = [KV, BV, P, I, F, P, P, P, P, P, SZ, P]
    lib.fastocr_focal_score_topk.restype = I
    lib.fastocr_focal_score_topk.argtypes = [KV, BV, P, I, F, D, P, P, P, P, I64, P, P, P, P, SZ, P]
    lib.fastocr_focal_attn_score_topk.restype = I
    lib.fastocr_focal_attn_score_topk.argtypes = [KV, BV, P, I, F, D, P, P, P, P, I64, P, P, P, P, P, SZ, P]
    lib.fastocr_kernel_timer_enable.restype, lib.fastocr_kernel_timer_enable.argtypes = I, [I, I]
    lib.fastocr_kernel_timer_read.restype, lib.fastocr_kernel_timer_read.argtypes = I, [I, P, I]
    lib.fastocr_select_focal_layers.restype = I
    lib.fastocr_select_focal_layers.argtypes = [P, I, I, I, ctypes.c_double, I, P, P]
    lib.fastocr_stream_probe.restype, lib.fastocr_stream_probe.argtypes = I, [P, P, SZ, P, P]
    lib.fastocr_set_tuning.restype, lib.fastocr_set_tuning.argtypes = I, [ctypes.c_char_p, I]
    lib.fastocr_exchange_timeouts.restype, lib.fastocr_exchange_timeouts.argtypes = I, [ctypes.POINTER(ctypes.c_uint64)]
    lib.fastocr_stream_release.restype, lib.fastocr_stream_release.argtypes = I, [P]
    lib.fastocr_strerror.restype, lib.fastocr_strerror.argtypes = ctypes.c_char_p, [I]
    lib.fastocr_version.restype, lib.fastocr_version.argtypes = ctypes.c_char_p, []
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().fastocr_strerror(int(status)).decode()


def version() -> str:
    return load_library().fastocr_version().decode()


def keep_count(n_visual: int, tau: float) -> int:
    return int(load_library().fastocr_keep_count(int(n_visual), float(tau)))


def set_tuning(key: str, value: int) -> None:
    rc = load_library().fastocr_set_tuning(key.encode(), int(value))
    if rc != OK:
        raise FastOcrError(rc, f"fastocr_set_tuning({key})")


def _ptr(t: Optional[torch.Tensor]):
    # the entry points' argtypes are declared, so a plain address converts (None is NULL)
    return None if t is None else t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported cache dtype {t.dtype}")


@dataclass
class KvCache:
    """One layer's cache: device tensors plus the strides that describe them.

    Contiguous: k, v of shape [B, Hkv, S, d] ("bhsd") or [B, S, Hkv, d] ("bshd").
    Paged: k, v of shape [n_pages, Hkv, page_tokens, d] and block_table int32 [B, max_pages].
    """
    k: torch.Tensor
    v: torch.Tensor
    layout: str = "bhsd"
    block_table: Optional[torch.Tensor] = None

    def view(self) -> KvView:
        """The C view of the cache.  Built once and kept while the tensors stay what they were
        (same addresses, shapes and strides): building it costs more host time than a small launch."""
        k, v, bt = self.k, self.v, self.block_table
        key = (k.data_ptr(), v.data_ptr(), k.shape, k.stride(), self.layout,
               None if bt is None else (bt.data_ptr(), bt.shape))
        cached = self.__dict__.get("_view")
        if cached is not None and cached[0] == key:
            return cached[1]
        view = self._build_view()
        self.__dict__["_view"] = (key, view)
        return view

    def _build_view(self) -> KvView:
        k, v = self.k, self.v
        assert k.shape == v.shape and k.dtype == v.dtype and k.stride() == v.stride()
        assert k.stride(-1) == 1
        if self.block_table is not None:
            n_pages, H, pt, d = k.shape
            bt = self.block_table
            assert bt.dtype == torch.int32 and bt.is_contiguous()
            return KvView(k.data_ptr(), v.data_ptr(), _dtype_code(k), H, d, k.stride(2), k.stride(1), 0,
                          pt, k.stride(0), bt.data_ptr(), bt.shape[1])
        if self.layout == "bhsd":
            B, H, S, d = k.shape
            return KvView(k.data_ptr(), v.data_ptr(), _dtype_code(k), H, d, k.stride(2), k.stride(1),
                          k.stride(0), 0, 0, None, 0)
        if self.layout == "bshd":
            B, S, H, d = k.shape
            return KvView(k.data_ptr(), v.data_ptr(), _dtype_code(k), H, d, k.stride(1), k.stride(2),
                          k.stride(0), 0, 0, None, 0)
        raise ValueError(self.layout)


@dataclass
class SeqBatch:
    """Per-sequence geometry: int32 device arrays and the host-side maxima."""
    seq_len: torch.Tensor
    vis_start: torch.Tensor
    vis_len: torch.Tensor
    max_seq_len: int
    max_vis_len: int

    @staticmethod
    def from_lists(seq_len, vis_start, vis_len, device) -> "SeqBatch":
        mk = lambda a: torch.tensor(list(a), dtype=torch.int32, device=device)
        return SeqBatch(mk(seq_len), mk(vis_start), mk(vis_len), max(seq_len) if len(seq_len) else 0,
                        max(vis_len) if len(vis_len) else 0)

    def view(self) -> BatchView:
        """The C view of the batch; kept while the arrays and the maxima stay what they were."""
        a, b, c = self.seq_len, self.vis_start, self.vis_len
        key = (a.data_ptr(), b.data_ptr(), c.data_ptr(), a.shape, self.max_seq_len, self.max_vis_len)
        cached = self.__dict__.get("_view")
        if cached is not None and cached[0] == key:
            return cached[1]
        for t in (a, b, c):
            assert t.dtype == torch.int32 and t.is_contiguous() and t.shape == a.shape
        view = BatchView(a.shape[0], a.data_ptr(), b.data_ptr(), c.data_ptr(), int(self.max_seq_len), int(self.max_vis_len))
        self.__dict__["_view"] = (key, view)
        return view


def _stream_handle(stream: Optional[torch.cuda.Stream]):
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream or None          # the default stream's handle is 0 = NULL


def workspace_bytes(op: int, cache: Optional[KvCache], batch: SeqBatch, n_q_heads: int, kmax: int = 0) -> int:
    lib = load_library()
    kv = cache.view() if cache is not None else None
    bv = batch.view()
    return int(lib.fastocr_workspace_bytes(op, ctypes.byref(kv) if kv is not None else None,
                                           ctypes.byref(bv), int(n_q_heads), int(kmax)))


class Workspace:
    """A reusable device scratch buffer (grown on demand, 256-byte aligned by torch)."""

    def __init__(self, device):
        self.device = device
        self.buf: Optional[torch.Tensor] = None

    def get(self, nbytes: int) -> torch.Tensor:
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        return self.buf


def _check(rc: int, what: str):
    if rc != OK:
        raise FastOcrError(rc, what)


def focal_score(cache: KvCache, batch: SeqBatch, q: torch.Tensor, scale: float, scores: torch.Tensor,
                ws: torch.Tensor, lse: Optional[torch.Tensor] = None,
                img_mass: Optional[torch.Tensor] = None, stream=None) -> None:
    """fastocr_focal_score: q [B,Hq,d]; scores fp32 [B, max_vis_len] (written in place)."""
    lib = load_library()
    kv, bv = cache.view(), batch.view()
    assert q.is_contiguous() and scores.is_contiguous() and scores.dtype == torch.float32
    assert scores.shape[0] == bv.batch and (scores.shape[1] == bv.max_vis_len or bv.batch == 0)
    _check(lib.fastocr_focal_score(ctypes.byref(kv), ctypes.byref(bv), _ptr(q), q.shape[1], float(scale),
                                   _ptr(scores), _ptr(lse), _ptr(img_mass), _ptr(ws), ws.numel(),
                                   _stream_handle(stream)), "fastocr_focal_score")


def topk_fixation(scores: torch.Tensor, batch: SeqBatch, tau: float, sel_idx: torch.Tensor,
                  sel_cnt: torch.Tensor, ws: Optional[torch.Tensor] = None,
                  prev_idx: Optional[torch.Tensor] = None, prev_cnt: Optional[torch.Tensor] = None,
                  stream=None) -> None:
    """fastocr_topk_fixation: sel_idx int32 [B,kmax], sel_cnt int32 [B] (written in place)."""
    lib = load_library()
    bv = batch.view()
    assert sel_idx.dtype == torch.int32 and sel_idx.is_contiguous() and sel_cnt.dtype == torch.int32
    assert scores.dtype == torch.float32 and scores.is_contiguous()
    assert scores.shape[1] == bv.max_vis_len or bv.batch == 0
    if prev_idx is not None:
        assert prev_idx.shape == sel_idx.shape and prev_idx.dtype == torch.int32 and prev_idx.is_contiguous()
    _check(lib.fastocr_topk_fixation(_ptr(scores), ctypes.byref(bv), float(tau), _ptr(prev_idx),
                                     _ptr(prev_cnt), _ptr(sel_idx), _ptr(sel_cnt), sel_idx.shape[1],
                                     _ptr(ws), 0 if ws is None else ws.numel(), _stream_handle(stream)),
           "fastocr_topk_fixation")


def sparse_decode_attn(cache: KvCache, batch: SeqBatch, q: torch.Tensor, scale: float,
                       sel_idx: torch.Tensor, sel_cnt: torch.Tensor, out: torch.Tensor,
                       ws: torch.Tensor, stream=None) -> None:
    """fastocr_sparse_decode_attn: out [B,Hq,d] in the cache dtype (written in place)."""
    lib = load_library()
    kv, bv = cache.view(), batch.view()
    assert q.is_contiguous() and out.is_contiguous() and out.shape == q.shape and out.dtype == q.dtype
    assert sel_idx.dtype == torch.int32 and sel_idx.is_contiguous() and sel_cnt.dtype == torch.int32
    _check(lib.fastocr_sparse_decode_attn(ctypes.byref(kv), ctypes.byref(bv), _ptr(q), q.shape[1],
                                          float(scale), _ptr(sel_idx), _ptr(sel_cnt), sel_idx.shape[1],
                                          _ptr(out), _ptr(ws), ws.numel(), _stream_handle(stream)),
           "fastocr_sparse_decode_attn")


def dense_decode_attn(cache: KvCache, batch: SeqBatch, q: torch.Tensor, scale: float, out: torch.Tensor,
                      ws: torch.Tensor, lse: Optional[torch.Tensor] = None, stream=None) -> None:
    """fastocr_dense_decode_attn: out [B,Hq,d] in the cache dtype (written in place)."""
    lib = load_library()
    kv, bv = cache.view(), batch.view()
    assert q.is_contiguous() and out.is_contiguous() and out.shape == q.shape and out.dtype == q.dtype
    _check(lib.fastocr_dense_decode_attn(ctypes.byref(kv), ctypes.byref(bv), _ptr(q), q.shape[1],
                                         float(scale), _ptr(out), _ptr(lse), _ptr(ws), ws.numel(),
                                         _stream_handle(stream)), "fastocr_dense_decode_attn")


def dense_decode_attn_static(cache: KvCache, batch: SeqBatch, q: torch.Tensor, scale: float, out: torch.Tensor,
                             lse: Optional[torch.Tensor] = None, stream=None) -> None:
    """fastocr_dense_decode_attn_static: as dense_decode_attn, scratch in the library's static device buffer."""
    lib = load_library()
    kv, bv = cache.view(), batch.view()
    assert q.is_contiguous() and out.is_contiguous() and out.shape == q.shape and out.dtype == q.dtype
    _check(lib.fastocr_dense_decode_attn_static(ctypes.byref(kv), ctypes.byref(bv), _ptr(q), q.shape[1],
                                                float(scale), _ptr(out), _ptr(lse), _stream_handle(stream)),
           "fastocr_dense_decode_attn_static")


def focal_attn_score(cache: KvCache, batch: SeqBatch, q: torch.Tensor, scale: float, out: torch.Tensor,
                     scores: torch.Tensor, ws: torch.Tensor, lse: Optional[torch.Tensor] = None,
                     img_mass: Optional[torch.Tensor] = None, stream=None) -> None:
    """fastocr_focal_attn_score: dense output [B,Hq,d] and scores fp32 [B, max_vis_len] in one call."""
    lib = load_library()
    kv, bv = cache.view(), batch.view()
    assert q.is_contiguous() and out.is_contiguous() and out.shape == q.shape and out.dtype == q.dtype
    assert scores.is_contiguous() and scores.dtype == torch.float32
    assert scores.shape[0] == bv.batch and (scores.shape[1] == bv.max_vis_len or bv.batch == 0)
    _check(lib.fastocr_focal_attn_score(ctypes.byref(kv), ctypes.byref(bv), _ptr(q), q.shape[1], float(scale),
                                        _ptr(out), _ptr(scores), _ptr(lse), _ptr(img_mass), _ptr(ws), ws.numel(),
                                        _stream_handle(stream)), "fastocr_focal_attn_score")


def focal_score_topk(cache: KvCache, batch: SeqBatch, q: torch.Tensor, scale: float, tau: float, scores: torch.Tensor,
                     sel_idx: torch.Tensor, sel_cnt: torch.Tensor, ws: torch.Tensor,
                     prev_idx: Optional[torch.Tensor] = None, prev_cnt: Optional[torch.Tensor] = None,
                     lse: Optional[torch.Tensor] = None, img_mass: Optional[torch.Tensor] = None, stream=None) -> None:
    """fastocr_focal_score_topk: scores and the selected set from one call."""
    lib = load_library()
    kv, bv = cache.view(), batch.view()
    assert q.is_contiguous() and scores.is_contiguous() and scores.dtype == torch.float32
    assert scores.shape[0] == bv.batch and (scores.shape[1] == bv.max_vis_len or bv.batch == 0)
    assert sel_idx.dtype == torch.int32 and sel_idx.is_contiguous() and sel_cnt.dtype == torch.int32
    if prev_idx is not None:
        assert prev_idx.shape == sel_idx.shape and prev_idx.dtype == torch.int32 and prev_idx.is_contiguous()
    _check(lib.fastocr_focal_score_topk(ctypes.byref(kv), ctypes.byref(bv), _ptr(q), q.shape[1], float(scale), float(tau),
                                        _ptr(prev_idx), _ptr(prev_cnt), _ptr(sel_idx), _ptr(sel_cnt), sel_idx.shape[1],
                                        _ptr(scores), _ptr(lse), _ptr(img_mass), _ptr(ws), ws.numel(),
                                        _stream_handle(stream)), "fastocr_focal_score_topk")


def focal_attn_score_topk(cache: KvCache, batch: SeqBatch, q: torch.Tensor, scale: float, tau: float, out: torch.Tensor,
                          scores: torch.Tensor, sel_idx: torch.Tensor, sel_cnt: torch.Tensor, ws: torch.Tensor,
                          prev_idx: Optional[torch.Tensor] = None, prev_cnt: Optional[torch.Tensor] = None,
                          lse: Optional[torch.Tensor] = None, img_mass: Optional[torch.Tensor] = None, stream=None) -> None:
    """fastocr_focal_attn_score_topk: a focal layer's dense output, its scores and the selected set from one call."""
    lib = load_library()
    kv, bv = cache.view(), batch.view()
    assert q.is_contiguous() and out.is_contiguous() and out.shape == q.shape and out.dtype == q.dtype
    assert scores.is_contiguous() and scores.dtype == torch.float32
    assert scores.shape[0] == bv.batch and (scores.shape[1] == bv.max_vis_len or bv.batch == 0)
    assert sel_idx.dtype == torch.int32 and sel_idx.is_contiguous() and sel_cnt.dtype == torch.int32
    if prev_idx is not None:
        assert prev_idx.shape == sel_idx.shape and prev_idx.dtype == torch.int32 and prev_idx.is_contiguous()
    _check(lib.fastocr_focal_attn_score_topk(ctypes.byref(kv), ctypes.byref(bv), _ptr(q), q.shape[1], float(scale), float(tau),
                                             _ptr(prev_idx), _ptr(prev_cnt), _ptr(sel_idx), _ptr(sel_cnt), sel_idx.shape[1],
                                             _ptr(out), _ptr(scores), _ptr(lse), _ptr(img_mass), _ptr(ws), ws.numel(),
                                             _stream_handle(stream)), "fastocr_focal_attn_score_topk")


def select_focal_layers(ratio, rho: float, gap: int):
    """fastocr_select_focal_layers on a host array [steps, layers, batch] (or [steps, layers])."""
    import numpy as np
    r = np.ascontiguousarray(np.asarray(ratio, dtype=np.float32))
    if r.ndim == 2:
        r = r[:, :, None]
    steps, layers, batch = r.shape
    out = np.zeros(layers, dtype=np.int32)
    n = ctypes.c_int32(0)
    _check(load_library().fastocr_select_focal_layers(r.ctypes.data, steps, layers, batch, float(rho), int(gap),
                                                      out.ctypes.data, ctypes.byref(n)), "fastocr_select_focal_layers")
    return [int(x) for x in out[: n.value]]


def stream_probe(src: torch.Tensor, dst: Optional[torch.Tensor], sink: torch.Tensor, stream=None) -> None:
    """fastocr_stream_probe: copy src to dst, or only read src when dst is None."""
    nbytes = src.numel() * src.element_size()
    _check(load_library().fastocr_stream_probe(_ptr(src), _ptr(dst), nbytes, _ptr(sink), _stream_handle(stream)),
           "fastocr_stream_probe")


def exchange_timeouts() -> int:
    """fastocr_exchange_timeouts: waves that gave up waiting inside a single-launch form since load."""
    n = ctypes.c_uint64(0)
    _check(load_library().fastocr_exchange_timeouts(ctypes.byref(n)), "fastocr_exchange_timeouts")
    return int(n.value)


def stream_release(stream: torch.cuda.Stream) -> None:
    """fastocr_stream_release: give back the exchange slots the stream holds (nothing of the library in flight on it)."""
    _check(load_library().fastocr_stream_release(stream.cuda_stream or None), "fastocr_stream_release")


def kernel_timer_enable(kernel: int, capacity: int) -> None:
    _check(load_library().fastocr_kernel_timer_enable(int(kernel), int(capacity)), "fastocr_kernel_timer_enable")


def kernel_timer_read(kernel: int, max_out: int = 65536):
    """Durations (ms) of the launches recorded since the last read."""
    buf = (ctypes.c_float * max_out)()
    n = load_library().fastocr_kernel_timer_read(int(kernel), buf, max_out)
    if n < 0:
        raise FastOcrError(n, "fastocr_kernel_timer_read")
    return [buf[i] for i in range(min(n, max_out))]
