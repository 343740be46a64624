"""FastOCR per-decode-step hot path for AMD MI355X (gfx950).

Hand-written HIP kernels behind a C ABI (include/fastocr.h, libfastocr.so); this package is
the thin Python binding (argument marshalling) plus the host-side step controller.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    FastOcrError, KvCache, SeqBatch, Workspace, dense_decode_attn, dense_decode_attn_static, focal_attn_score, focal_attn_score_topk, focal_score, focal_score_topk, keep_count,
    load_library, sparse_decode_attn, topk_fixation, workspace_bytes,
)
from .controller import FixationController  # noqa: F401
