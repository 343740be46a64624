"""CPU oracle of the FastOCR decode hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``fastocr_oracle.c`` (plain C, fp64).  Only the test
suite, ``__graft_entry__.smoke()`` and the benchmark's ``cpu_baseline`` leg may
import this package.  It shares no code with the HIP library and imports
nothing from it.

Arrays are numpy: fp32 caches as ``float32``, bf16 caches as ``uint16`` holding
the raw bf16 bit patterns (exactly the bits the GPU sees).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fastocr_oracle.c")
_LIB = os.path.join(_HERE, "libfastocr_oracle.so")

F32, BF16 = 0, 1


# FASTOCR_ORACLE_SANITIZE=1 (set by tests/test_host_sanitizers.py for a child process) builds and
# loads the same source under AddressSanitizer and UndefinedBehaviorSanitizer instead.
_SANITIZE = os.environ.get("FASTOCR_ORACLE_SANITIZE") == "1"
_LIB_SAN = os.path.join(_HERE, "libfastocr_oracle_san.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP for the outer head loop only)."""
    lib = _LIB_SAN if _SANITIZE else _LIB
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        tmp = lib + f".tmp{os.getpid()}"
        flags = ["-O2"]
        if _SANITIZE:
            flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
        subprocess.check_call(
            ["gcc", *flags, "-std=c99", "-fPIC", "-shared", "-fopenmp", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, lib)
    return lib


class _KV(ctypes.Structure):
    _fields_ = [
        ("k", ctypes.c_void_p),
        ("v", ctypes.c_void_p),
        ("dtype", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("stride_token", ctypes.c_int64),
        ("stride_head", ctypes.c_int64),
        ("stride_seq", ctypes.c_int64),
        ("page_tokens", ctypes.c_int32),
        ("stride_page", ctypes.c_int64),
        ("block_table", ctypes.c_void_p),
        ("max_pages_per_seq", ctypes.c_int32),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.orc_keep_count.restype = ctypes.c_int64
        lib.orc_keep_count.argtypes = [ctypes.c_int64, ctypes.c_double]
        lib.orc_focal_score.restype = ctypes.c_int
        lib.orc_focal_score.argtypes = [
            ctypes.POINTER(_KV), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
        ]
        lib.orc_topk.restype = ctypes.c_int64
        lib.orc_topk.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p]
        lib.orc_decode_attn.restype = ctypes.c_int
        lib.orc_decode_attn.argtypes = [
            ctypes.POINTER(_KV), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
        ]
        lib.orc_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


@dataclass
class Cache:
    """One layer's KV cache in host memory.

    Contiguous mode: ``k``/``v`` are arrays whose element strides are given by
    ``stride_seq / stride_token / stride_head`` (head_dim contiguous).
    Paged mode (``page_tokens > 0``): token j of sequence b lives in page
    ``block_table[b, j // page_tokens]`` at ``stride_page`` elements per page.
    """

    k: np.ndarray
    v: np.ndarray
    n_kv_heads: int
    head_dim: int
    stride_token: int
    stride_head: int
    stride_seq: int = 0
    page_tokens: int = 0
    stride_page: int = 0
    block_table: Optional[np.ndarray] = None

    @staticmethod
    def from_bhsd(k: np.ndarray, v: np.ndarray) -> "Cache":
        """k, v: C-contiguous [B, Hkv, S, d]."""
        B, H, S, d = k.shape
        return Cache(np.ascontiguousarray(k), np.ascontiguousarray(v), H, d,
                     stride_token=d, stride_head=S * d, stride_seq=H * S * d)

    @staticmethod
    def from_bshd(k: np.ndarray, v: np.ndarray) -> "Cache":
        """k, v: C-contiguous [B, S, Hkv, d]."""
        B, S, H, d = k.shape
        return Cache(np.ascontiguousarray(k), np.ascontiguousarray(v), H, d,
                     stride_token=H * d, stride_head=d, stride_seq=S * H * d)

    def _dtype_code(self) -> int:
        if self.k.dtype == np.float32:
            return F32
        if self.k.dtype == np.uint16:
            return BF16
        raise TypeError(f"cache dtype {self.k.dtype}: use float32 or uint16 (bf16 bits)")

    def _c(self) -> _KV:
        assert self.k.dtype == self.v.dtype
        bt = None
        mp = 0
        if self.page_tokens > 0:
            assert self.block_table is not None and self.block_table.dtype == np.int32
            assert self.block_table.flags.c_contiguous
            bt = self.block_table.ctypes.data
            mp = self.block_table.shape[1]
        return _KV(self.k.ctypes.data, self.v.ctypes.data, self._dtype_code(), self.n_kv_heads,
                   self.head_dim, self.stride_token, self.stride_head, self.stride_seq,
                   self.page_tokens, self.stride_page, bt, mp)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def max_threads() -> int:
    return int(_load().orc_max_threads())


def keep_count(n_visual: int, tau: float) -> int:
    """ceil(tau * N), the focal token set size (Sec. 3.1.2)."""
    return int(_load().orc_keep_count(int(n_visual), float(tau)))


def focal_score(cache: Cache, seq_len, vis_start, vis_len, q: np.ndarray, scale: float,
                n_threads: int = 1):
    """Head-averaged attention at image tokens (Eq. 1 / text under Eq. 2).

    q: [B, Hq, d] in the cache dtype.  Returns (scores [B, max_vis] f64 with
    rows zero beyond vis_len, lse [B, Hq] f64, img_mass [B] f64).
    """
    lib = _load()
    seq_len, vis_start, vis_len = _i32(seq_len), _i32(vis_start), _i32(vis_len)
    B, Hq, d = q.shape
    assert q.dtype == cache.k.dtype and d == cache.head_dim and q.flags.c_contiguous
    max_vis = int(vis_len.max()) if B else 0
    scores = np.zeros((B, max(max_vis, 1)), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64)
    mass = np.zeros((B,), dtype=np.float64)
    kv = cache._c()
    rc = lib.orc_focal_score(ctypes.byref(kv), B, seq_len.ctypes.data, vis_start.ctypes.data,
                             vis_len.ctypes.data, q.ctypes.data, Hq, float(scale),
                             scores.ctypes.data, scores.shape[1], lse.ctypes.data,
                             mass.ctypes.data, int(n_threads))
    if rc != 0:
        raise ValueError(f"orc_focal_score failed: {rc}")
    return scores[:, :max_vis], lse, mass


def topk(scores: np.ndarray, k: int) -> np.ndarray:
    """Exact top-k of one sequence's scores; ties to the lower index; ascending indices."""
    lib = _load()
    s = np.ascontiguousarray(np.asarray(scores, dtype=np.float64))
    n = s.shape[0]
    k = max(0, min(int(k), n))
    out = np.zeros((max(k, 1),), dtype=np.int32)
    got = lib.orc_topk(s.ctypes.data, n, k, out.ctypes.data)
    if got < 0:
        raise MemoryError
    return out[:got]


def topk_fixation(scores: np.ndarray, vis_len, tau: float):
    """Per-sequence TopK_{ceil(tau N_b)}; returns (sel_idx [B, kmax] int32, sel_cnt [B] int32).

    The previous step's set plays no part: a warm start must not change the result.
    """
    vis_len = _i32(vis_len)
    B = vis_len.shape[0]
    cnt = np.array([keep_count(int(n), tau) for n in vis_len], dtype=np.int32)
    kmax = max(int(cnt.max()) if B else 0, 1)
    idx = np.full((B, kmax), -1, dtype=np.int32)
    for b in range(B):
        sel = topk(scores[b, : vis_len[b]], int(cnt[b]))
        idx[b, : sel.shape[0]] = sel
    return idx, cnt


def decode_attn(cache: Cache, seq_len, vis_start, vis_len, q: np.ndarray, scale: float,
                sel_idx: Optional[np.ndarray] = None, sel_cnt=None, n_threads: int = 1):
    """Attention over the kept set T u F (sel_idx given) or the full cache (None). Eq. 2.

    Returns (out [B, Hq, d] f64, lse [B, Hq] f64).
    """
    lib = _load()
    seq_len, vis_start, vis_len = _i32(seq_len), _i32(vis_start), _i32(vis_len)
    B, Hq, d = q.shape
    assert q.dtype == cache.k.dtype and d == cache.head_dim and q.flags.c_contiguous
    out = np.zeros((B, Hq, d), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64)
    kv = cache._c()
    if sel_idx is None:
        sp, cp, kmax = None, None, 0
    else:
        sel_idx = _i32(sel_idx)
        sel_cnt = _i32(sel_cnt)
        assert sel_idx.ndim == 2 and sel_idx.shape[0] == B
        sp, cp, kmax = sel_idx.ctypes.data, sel_cnt.ctypes.data, sel_idx.shape[1]
    rc = lib.orc_decode_attn(ctypes.byref(kv), B, seq_len.ctypes.data, vis_start.ctypes.data,
                             vis_len.ctypes.data, q.ctypes.data, Hq, float(scale),
                             sp, cp, kmax, out.ctypes.data, lse.ctypes.data, int(n_threads))
    if rc != 0:
        raise ValueError(f"orc_decode_attn failed: {rc}")
    return out, lse
