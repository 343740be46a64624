"""Helpers of the GPU parity tests: run the HIP path through the C-ABI binding on inputs that
also go, bit for bit, to the CPU oracle, and compare to the stated bars.

Bars: image scores absolute 1e-6; attention outputs per row max|o - o_ref| / max|o_ref| <= 1e-5
(fp32 cache) or 2e-2 (bf16 cache); selected sets bit-exact on identical fp32 scores, and up to
ties within 1e-6 of the k-th score when each side scores for itself.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2605_17447_amd as fo
from paper_2605_17447_amd import binding as fb

DEV = "cuda:0"
SCORE_ATOL = 1e-6
OUT_RTOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


def to_np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


def from_np(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(DEV)
    return torch.from_numpy(a.copy()).to(DEV)


class GpuProblem:
    """Device-side twin of a host problem (k, v, q arrays + geometry)."""

    def __init__(self, k, v, q, seq_len, vis_start, vis_len, scale, layout="bhsd", block_table=None,
                 max_seq_len=None, max_vis_len=None):
        self.k, self.v, self.q = k, v, q                      # torch device tensors
        self.cache = fo.KvCache(k, v, layout, block_table)
        seq_len, vis_start, vis_len = (list(map(int, x)) for x in (seq_len, vis_start, vis_len))
        self.batch = fo.SeqBatch.from_lists(seq_len, vis_start, vis_len, DEV)
        if max_seq_len is not None:
            self.batch.max_seq_len = max_seq_len
        if max_vis_len is not None:
            self.batch.max_vis_len = max_vis_len
        self.B, self.Hq, self.d = q.shape
        self.scale = float(np.float32(scale))
        self.seq_len, self.vis_start, self.vis_len = seq_len, vis_start, vis_len
        self._ws = fo.Workspace(DEV)

    def ws(self, op, kmax=0):
        return self._ws.get(fo.workspace_bytes(op, self.cache if op != fb.OP_TOPK_FIXATION else None,
                                               self.batch, self.Hq, kmax))

    def scores(self, want_lse=False, want_mass=False):
        sc = torch.full((self.B, self.batch.max_vis_len), -7.0, dtype=torch.float32, device=DEV)
        lse = torch.zeros((self.B, self.Hq), dtype=torch.float32, device=DEV) if want_lse else None
        mass = torch.zeros((self.B,), dtype=torch.float32, device=DEV) if want_mass else None
        fo.focal_score(self.cache, self.batch, self.q, self.scale, sc, self.ws(fb.OP_FOCAL_SCORE), lse, mass)
        return sc, lse, mass

    def topk(self, scores, tau, prev_idx=None, prev_cnt=None, kmax=None, inplace=False):
        kmax = kmax or max(1, fo.keep_count(self.batch.max_vis_len, tau))
        if inplace:
            idx, cnt = prev_idx, prev_cnt
        else:
            idx = torch.full((self.B, kmax), -1, dtype=torch.int32, device=DEV)
            cnt = torch.full((self.B,), -1, dtype=torch.int32, device=DEV)
        fo.topk_fixation(scores, self.batch, tau, idx, cnt, self.ws(fb.OP_TOPK_FIXATION, kmax), prev_idx, prev_cnt)
        return idx, cnt

    def sparse(self, idx, cnt):
        out = torch.full_like(self.q, 3.0)
        fo.sparse_decode_attn(self.cache, self.batch, self.q, self.scale, idx, cnt, out,
                              self.ws(fb.OP_SPARSE_DECODE_ATTN, idx.shape[1]))
        return out

    def dense(self, want_lse=False):
        out = torch.full_like(self.q, 3.0)
        lse = torch.zeros((self.B, self.Hq), dtype=torch.float32, device=DEV) if want_lse else None
        fo.dense_decode_attn(self.cache, self.batch, self.q, self.scale, out, self.ws(fb.OP_DENSE_DECODE_ATTN), lse)
        return out, lse

    def focal_attn(self, want_lse=False, want_mass=False):
        """Dense output and scores from the one-call focal layer."""
        out = torch.full_like(self.q, 3.0)
        sc = torch.full((self.B, self.batch.max_vis_len), -7.0, dtype=torch.float32, device=DEV)
        lse = torch.zeros((self.B, self.Hq), dtype=torch.float32, device=DEV) if want_lse else None
        mass = torch.zeros((self.B,), dtype=torch.float32, device=DEV) if want_mass else None
        fo.focal_attn_score(self.cache, self.batch, self.q, self.scale, out, sc, self.ws(fb.OP_FOCAL_ATTN_SCORE),
                            lse, mass)
        return out, sc, lse, mass

    # ---- the same problem for the oracle -------------------------------------------------
    def oracle_cache(self) -> oracle.Cache:
        k, v = to_np(self.k), to_np(self.v)
        if self.cache.block_table is not None:
            n_pages, H, pt, d = k.shape
            return oracle.Cache(k, v, H, d, stride_token=d, stride_head=pt * d, page_tokens=pt,
                                stride_page=H * pt * d, block_table=self.cache.block_table.cpu().numpy())
        return oracle.Cache.from_bhsd(k, v) if self.cache.layout == "bhsd" else oracle.Cache.from_bshd(k, v)

    def oracle_args(self, sub=None):
        """(cache, seq_len, vis_start, vis_len, q, scale) for all sequences."""
        return (self.oracle_cache(), self.seq_len, self.vis_start, self.vis_len, to_np(self.q), self.scale)


def problem_from_case(case, layout="bhsd") -> GpuProblem:
    """case: tests.util.TinyCase (numpy, [B,Hkv,S,d])."""
    k, v, q = from_np(case.k), from_np(case.v), from_np(case.q)
    if layout == "bshd":
        k = k.permute(0, 2, 1, 3).contiguous()
        v = v.permute(0, 2, 1, 3).contiguous()
    return GpuProblem(k, v, q, case.seq_len, case.vis_start, case.vis_len, case.scale, layout)


def row_rel_err(out: torch.Tensor, ref: np.ndarray) -> float:
    o = out.detach().float().cpu().numpy().astype(np.float64)
    num = np.abs(o - ref).max(axis=-1)
    den = np.maximum(np.abs(ref).max(axis=-1), 1e-30)
    return float((num / den).max()) if num.size else 0.0


def check_out(out: torch.Tensor, ref: np.ndarray, what=""):
    err = row_rel_err(out, ref)
    tol = OUT_RTOL[out.dtype]
    assert np.isfinite(out.float().cpu().numpy()).all(), f"{what}: non-finite output"
    assert err <= tol, f"{what}: row-relative error {err:.3e} > {tol:.1e}"
    return err


def check_scores(sc: torch.Tensor, ref: np.ndarray, vis_len, what=""):
    got = sc.detach().cpu().numpy().astype(np.float64)
    worst = 0.0
    for b, n in enumerate(vis_len):
        if n:
            worst = max(worst, float(np.abs(got[b, :n] - ref[b, :n]).max()))
    assert worst <= SCORE_ATOL, f"{what}: score error {worst:.3e} > {SCORE_ATOL:.0e}"
    return worst


def check_set_valid(idx_row: np.ndarray, cnt: int, ref_scores: np.ndarray, k: int, what=""):
    """A selected set against scores the oracle computed itself: exact size, ascending and
    distinct, holds everything clearly above the k-th score and nothing clearly below it."""
    assert cnt == k, f"{what}: count {cnt} != {k}"
    a = idx_row[:k].astype(np.int64)
    if k == 0:
        return
    assert np.all(np.diff(a) > 0), f"{what}: indices not strictly ascending"
    assert a[0] >= 0 and a[-1] < ref_scores.shape[0], f"{what}: index out of range"
    s_k = np.sort(ref_scores)[::-1][k - 1]
    must = np.nonzero(ref_scores > s_k + 1e-6)[0]
    assert np.isin(must, a).all(), f"{what}: a token clearly above the threshold is missing"
    assert ref_scores[a].min() >= s_k - 1e-6, f"{what}: a token clearly below the threshold was taken"
