"""Pins of the CPU oracle against things other than itself (CPU only).

Each test is chosen so that a plausible mistake in oracle/fastocr_oracle.c -- a
dropped term, a wrong head mapping, a transposed operand, softmax over the wrong
set, a wrong tie rule or rounding of ceil(tau N) -- fails at least one of them.
"""
from fractions import Fraction
import math
import os

import numpy as np
import pytest
import torch

import oracle
from util import (TinyCase, as_f64, brute_attn, brute_logits, brute_scores, brute_topk, store)

HEAD_COMBOS = [(1, 1), (2, 1), (4, 1), (4, 2), (6, 3), (8, 8), (7, 1), (12, 4)]


def _cache(case):
    return oracle.Cache.from_bhsd(case.k, case.v)


def _scores(case, **kw):
    return oracle.focal_score(_cache(case), case.seq_len, case.vis_start, case.vis_len, case.q,
                              case.scale, **kw)


# ----------------------------------------------------------------- brute force

@pytest.mark.parametrize("Hq,Hkv", HEAD_COMBOS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scores_match_pure_python_brute_force(Hq, Hkv, dtype):
    case = TinyCase(seed=Hq * 31 + Hkv, B=2, Hq=Hq, Hkv=Hkv, d=8, n_vis=[23, 40], pre=[3, 0],
                    post=[5, 2], dtype=dtype)
    sc, lse, mass = _scores(case)
    for b in range(case.B):
        ref = brute_scores(case, b)
        n = int(case.vis_len[b])
        assert np.allclose(sc[b, :n], ref, rtol=1e-12, atol=1e-15)
        assert abs(mass[b] - math.fsum(ref)) < 1e-12
        # the per-head log-sum-exp the call also returns: ln sum_j exp(logit_j) over ALL cached tokens
        # (image and text), from the pure-Python logits
        for h in range(Hq):
            lg = brute_logits(case, b, h)
            mx = max(lg)
            want = mx + math.log(math.fsum(math.exp(x - mx) for x in lg))
            assert abs(lse[b, h] - want) <= 1e-12 * max(1.0, abs(want))


@pytest.mark.parametrize("Hq,Hkv", HEAD_COMBOS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_matches_pure_python_brute_force(Hq, Hkv, dtype):
    case = TinyCase(seed=1000 + Hq * 31 + Hkv, B=2, Hq=Hq, Hkv=Hkv, d=6, n_vis=[17, 30], pre=[4, 1],
                    post=[2, 6], dtype=dtype)
    cache = _cache(case)
    dense, _ = oracle.decode_attn(cache, case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)
    sel = np.array([[0, 5, 16, -1, -1], [29, 3, 7, 11, 2]], np.int32)     # second row unsorted on purpose
    cnt = np.array([3, 5], np.int32)
    sparse, _ = oracle.decode_attn(cache, case.seq_len, case.vis_start, case.vis_len, case.q, case.scale,
                                   sel, cnt)
    for b in range(case.B):
        for h in range(Hq):
            assert np.allclose(dense[b, h], brute_attn(case, b, h, None), rtol=1e-12, atol=1e-14)
            s = [int(x) for x in sel[b, : cnt[b]]]
            assert np.allclose(sparse[b, h], brute_attn(case, b, h, s), rtol=1e-12, atol=1e-14)


def test_topk_matches_sorted_brute_force_with_ties():
    rng = np.random.default_rng(7)
    for n, k in [(1, 1), (5, 0), (5, 5), (64, 13), (257, 40), (1000, 999)]:
        s = rng.integers(0, 12, size=n).astype(np.float64) / 8.0       # many exact ties
        got = oracle.topk(s, k)
        assert got.tolist() == brute_topk(s.tolist(), k)
        assert len(got) == k and np.all(np.diff(got) > 0)


def test_topk_tie_goes_to_lower_index():
    s = np.array([0.5, 0.25, 0.5, 0.5, 0.125])
    assert oracle.topk(s, 2).tolist() == [0, 2]
    assert oracle.topk(s, 3).tolist() == [0, 2, 3]
    assert oracle.topk(s, 4).tolist() == [0, 1, 2, 3]


# --------------------------------------------------------------- closed forms

def test_probabilities_sum_to_one_and_image_mass_is_eq1_ratio():
    # Eq. 1: r = sum_I a / (sum_I a + sum_T a); with the softmax over I u T the denominator is 1.
    case = TinyCase(seed=3, B=3, Hq=4, Hkv=2, d=8, n_vis=[16, 9, 25], pre=[4, 0, 2], post=[3, 5, 0])
    sc, lse, mass = _scores(case)
    for b in range(3):
        assert 0.0 < mass[b] < 1.0
        assert abs(sc[b, : case.vis_len[b]].sum() - mass[b]) < 1e-14
    # no text at all -> all mass on the image
    case2 = TinyCase(seed=4, B=1, Hq=2, Hkv=1, d=4, n_vis=11, pre=0, post=0)
    assert abs(_scores(case2)[2][0] - 1.0) < 1e-14
    # text mass from a complementary call: treat text-after as the "image"
    tot = mass[0]
    c = _cache(case)
    pre, n, post = 4, 16, 3
    s_pre, _, m_pre = oracle.focal_score(c, case.seq_len[:1], [0], [pre], case.q[:1], case.scale)
    s_post, _, m_post = oracle.focal_score(c, case.seq_len[:1], [pre + n], [post], case.q[:1], case.scale)
    assert abs(tot + m_pre[0] + m_post[0] - 1.0) < 1e-13


def test_identical_keys_give_uniform_scores_and_mean_of_values():
    case = TinyCase(seed=5, B=1, Hq=4, Hkv=2, d=8, n_vis=20, pre=3, post=2)
    case.k[:] = case.k[:, :, :1, :]                        # every token has the same key
    sc, lse, mass = _scores(case)
    S = int(case.seq_len[0])
    assert np.allclose(sc[0], 1.0 / S, rtol=1e-13)
    sel = np.array([[2, 9, 17]], np.int32); cnt = np.array([3], np.int32)
    out, _ = oracle.decode_attn(_cache(case), case.seq_len, case.vis_start, case.vis_len, case.q,
                                case.scale, sel, cnt)
    kept = [0, 1, 2, 3 + 2, 3 + 9, 3 + 17, 23, 24]
    V = as_f64(case.v)
    for h in range(4):
        assert np.allclose(out[0, h], V[0, h // 2, kept].mean(axis=0), rtol=1e-13, atol=1e-15)


def test_planted_key_takes_all_the_mass():
    case = TinyCase(seed=6, B=1, Hq=3, Hkv=1, d=8, n_vis=30, pre=2, post=2)
    Q = as_f64(case.q)[0]
    qbar = Q.mean(axis=0)
    # a key far along every head's query direction: sum of unit queries, scaled up
    dirn = sum(Q[h] / np.linalg.norm(Q[h]) for h in range(3))
    assert all(Q[h] @ dirn > 0.3 * np.linalg.norm(Q[h]) for h in range(3)), "case must be well posed"
    case.k[0, 0, 2 + 11] = (dirn * 400.0).astype(np.float32)
    sc, _, mass = _scores(case)
    assert sc[0, 11] > 1.0 - 1e-9 and abs(mass[0] - sc[0].sum()) < 1e-14
    assert oracle.topk(sc[0], 1).tolist() == [11]


def test_softmax_shift_invariance_exact_on_dyadic_inputs():
    rng = np.random.default_rng(8)
    B, Hq, Hkv, d, S = 1, 4, 2, 8, 24
    k = rng.integers(-16, 17, size=(B, Hkv, S, d)).astype(np.float32) / 16
    v = rng.integers(-16, 17, size=(B, Hkv, S, d)).astype(np.float32) / 16
    q = rng.integers(-16, 17, size=(B, Hq, d)).astype(np.float32) / 16
    u = rng.integers(-32, 33, size=(1, Hkv, 1, d)).astype(np.float32) / 16
    a = oracle.focal_score(oracle.Cache.from_bhsd(k, v), [S], [4], [15], q, 0.25)[0]
    b = oracle.focal_score(oracle.Cache.from_bhsd(k + u, v), [S], [4], [15], q, 0.25)[0]
    assert np.allclose(a, b, rtol=1e-12)


def test_gqa_equals_mha_with_replicated_kv_heads():
    case = TinyCase(seed=9, B=2, Hq=6, Hkv=2, d=8, n_vis=[12, 20], pre=[2, 3], post=[4, 1], dtype="bf16")
    rep_k = np.repeat(case.k, 3, axis=1)
    rep_v = np.repeat(case.v, 3, axis=1)
    a = _scores(case)[0]
    mha = oracle.Cache.from_bhsd(rep_k, rep_v)
    b = oracle.focal_score(mha, case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)[0]
    assert np.array_equal(a, b)
    oa = oracle.decode_attn(_cache(case), case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)[0]
    ob = oracle.decode_attn(mha, case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)[0]
    assert np.array_equal(oa, ob)


def test_scale_is_applied_to_logits():
    # with one head and two tokens the score is a logistic function of scale * (q.k0 - q.k1)
    k = np.zeros((1, 1, 2, 4), np.float32); v = np.zeros_like(k)
    q = np.array([[[1.0, 2.0, 0.0, -1.0]]], np.float32)
    k[0, 0, 0] = [0.5, 0.25, 3.0, 0.0]     # q.k0 = 1.0
    k[0, 0, 1] = [0.0, 0.0, 1.0, 2.0]      # q.k1 = -2.0
    for scale in (1.0, 0.5, 0.125):
        sc = oracle.focal_score(oracle.Cache.from_bhsd(k, v), [2], [0], [2], q, scale)[0]
        assert abs(sc[0, 0] - 1.0 / (1.0 + math.exp(-3.0 * scale))) < 1e-15


# ------------------------------------------------ library routine cross-check

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_equals_library_sdpa_on_gathered_rows(dtype):
    case = TinyCase(seed=11, B=2, Hq=8, Hkv=2, d=16, n_vis=[40, 64], pre=[5, 0], post=[7, 9], dtype=dtype)
    cache = _cache(case)
    sc, _, _ = _scores(case)
    sel, cnt = oracle.topk_fixation(sc, case.vis_len, 0.25)
    out, lse = oracle.decode_attn(cache, case.seq_len, case.vis_start, case.vis_len, case.q, case.scale,
                                  sel, cnt)
    K, V, Q = (torch.from_numpy(as_f64(x)) for x in (case.k, case.v, case.q))
    for b in range(case.B):
        S, N, v0 = int(case.seq_len[b]), int(case.vis_len[b]), int(case.vis_start[b])
        J = list(range(v0)) + [v0 + int(i) for i in sel[b, : cnt[b]]] + list(range(v0 + N, S))
        kb = K[b][:, J].repeat_interleave(4, dim=0)                     # [Hq, |J|, d]
        vb = V[b][:, J].repeat_interleave(4, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(
            Q[b].unsqueeze(1), kb, vb, scale=case.scale).squeeze(1)
        assert np.allclose(out[b], ref.numpy(), rtol=1e-11, atol=1e-13)
        ref_lse = torch.logsumexp(torch.einsum("hd,hjd->hj", Q[b], kb) * case.scale, dim=-1)
        assert np.allclose(lse[b], ref_lse.numpy(), rtol=1e-12)


# ------------------------------------------------------------ method invariants

def test_tau_one_is_dense_and_tau_zero_is_text_only():
    case = TinyCase(seed=12, B=2, Hq=4, Hkv=2, d=8, n_vis=[18, 31], pre=[3, 2], post=[4, 0], dtype="bf16")
    cache = _cache(case)
    args = (cache, case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)
    sc = oracle.focal_score(*args)[0]
    dense, dlse = oracle.decode_attn(*args)
    sel, cnt = oracle.topk_fixation(sc, case.vis_len, 1.0)
    assert cnt.tolist() == [18, 31] and sel[1].tolist() == list(range(31))
    full, flse = oracle.decode_attn(*args, sel, cnt)
    assert np.allclose(full, dense, rtol=1e-13, atol=1e-15) and np.allclose(flse, dlse, rtol=1e-13)
    # tau = 0: the visual span is cut out of the cache
    sel0, cnt0 = oracle.topk_fixation(sc, case.vis_len, 0.0)
    assert cnt0.tolist() == [0, 0]
    text_only, _ = oracle.decode_attn(*args, sel0, cnt0)
    for b in range(2):
        S, N, v0 = int(case.seq_len[b]), int(case.vis_len[b]), int(case.vis_start[b])
        keep = list(range(v0)) + list(range(v0 + N, S))
        cut = oracle.Cache.from_bhsd(case.k[b:b + 1][:, :, keep], case.v[b:b + 1][:, :, keep])
        ref, _ = oracle.decode_attn(cut, [len(keep)], [0], [0], case.q[b:b + 1], case.scale)
        assert np.allclose(text_only[b], ref[0], rtol=1e-13, atol=1e-15)


def test_selection_is_permutation_invariant_and_output_unchanged():
    case = TinyCase(seed=13, B=1, Hq=4, Hkv=2, d=8, n_vis=48, pre=4, post=4)
    args = lambda c: (oracle.Cache.from_bhsd(c.k, c.v), c.seq_len, c.vis_start, c.vis_len, c.q, c.scale)
    sc = oracle.focal_score(*args(case))[0]
    sel, cnt = oracle.topk_fixation(sc, case.vis_len, 0.2)
    out, _ = oracle.decode_attn(*args(case), sel, cnt)
    perm = np.random.default_rng(1).permutation(48)              # new position p holds old token perm[p]
    pc = TinyCase(seed=13, B=1, Hq=4, Hkv=2, d=8, n_vis=48, pre=4, post=4)
    pc.k[:, :, 4:52] = case.k[:, :, 4 + perm]
    pc.v[:, :, 4:52] = case.v[:, :, 4 + perm]
    sc2 = oracle.focal_score(*args(pc))[0]
    sel2, cnt2 = oracle.topk_fixation(sc2, pc.vis_len, 0.2)
    assert sorted(perm[sel2[0, : cnt2[0]]].tolist()) == sel[0, : cnt[0]].tolist()
    out2, _ = oracle.decode_attn(*args(pc), sel2, cnt2)
    assert np.allclose(out, out2, rtol=1e-12, atol=1e-14)


def test_selected_sets_nest_as_tau_grows():
    case = TinyCase(seed=14, B=1, Hq=2, Hkv=1, d=8, n_vis=200, pre=3, post=3)
    sc = _scores(case)[0]
    prev = set()
    for tau in (0.02, 0.05, 0.1, 0.25, 0.5, 1.0):
        sel, cnt = oracle.topk_fixation(sc, case.vis_len, tau)
        cur = set(sel[0, : cnt[0]].tolist())
        assert len(cur) == math.ceil(Fraction(str(tau)) * 200) and prev <= cur
        prev = cur


def test_lse_merge_identity_pins_the_split_reduction():
    # Attn(A u B) = (e^{lA} oA + e^{lB} oB) / (e^{lA} + e^{lB}) with l the log-sum-exp of each part
    case = TinyCase(seed=15, B=1, Hq=4, Hkv=2, d=8, n_vis=40, pre=0, post=0)
    args = (_cache(case), case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)
    A = np.arange(0, 40, 3, dtype=np.int32); Bset = np.array([i for i in range(40) if i % 3], np.int32)
    oa, la = oracle.decode_attn(*args, A[None], [len(A)])
    ob, lb = oracle.decode_attn(*args, Bset[None], [len(Bset)])
    full, lf = oracle.decode_attn(*args)
    wa = np.exp(la - lf)[..., None]; wb = np.exp(lb - lf)[..., None]
    assert np.allclose(wa * oa + wb * ob, full, rtol=1e-12, atol=1e-14)
    assert np.allclose(np.logaddexp(la, lb), lf, rtol=1e-13)


def test_output_does_not_depend_on_index_order():
    case = TinyCase(seed=16, B=1, Hq=2, Hkv=2, d=8, n_vis=30, pre=2, post=2)
    args = (_cache(case), case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)
    a, _ = oracle.decode_attn(*args, np.array([[1, 4, 9, 20]], np.int32), [4])
    b, _ = oracle.decode_attn(*args, np.array([[20, 1, 9, 4]], np.int32), [4])
    assert np.allclose(a, b, rtol=1e-13, atol=1e-16)


def test_paged_and_token_major_layouts_equal_contiguous():
    case = TinyCase(seed=17, B=2, Hq=4, Hkv=2, d=8, n_vis=[20, 33], pre=[2, 5], post=[3, 1], dtype="bf16")
    ref_s = _scores(case)[0]
    ref_o = oracle.decode_attn(_cache(case), case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)[0]
    # [B, S, Hkv, d]
    tm = oracle.Cache.from_bshd(case.k.transpose(0, 2, 1, 3), case.v.transpose(0, 2, 1, 3))
    assert np.array_equal(oracle.focal_score(tm, case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)[0], ref_s)
    # pages of 8 tokens, scattered through one pool
    pt, S = 8, case.S
    n_pages = -(-S // pt)
    table = np.random.default_rng(2).permutation(2 * n_pages).astype(np.int32).reshape(2, n_pages)
    pool_k = np.zeros((2 * n_pages, 2, pt, 8), case.k.dtype); pool_v = np.zeros_like(pool_k)
    for b in range(2):
        for j in range(S):
            pool_k[table[b, j // pt], :, j % pt] = case.k[b, :, j]
            pool_v[table[b, j // pt], :, j % pt] = case.v[b, :, j]
    paged = oracle.Cache(pool_k, pool_v, 2, 8, stride_token=8, stride_head=pt * 8, page_tokens=pt,
                         stride_page=2 * pt * 8, block_table=table)
    assert np.array_equal(oracle.focal_score(paged, case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)[0], ref_s)
    assert np.array_equal(oracle.decode_attn(paged, case.seq_len, case.vis_start, case.vis_len, case.q, case.scale)[0], ref_o)


# ------------------------------------------------------------------ ceil(tau N)

def _golden_keep_counts():
    path = os.path.join(os.path.dirname(__file__), "golden", "keep_counts.txt")
    rows = []
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            n, tau, k = line.split()
            rows.append((int(n), tau, int(k)))
    return rows


def test_keep_count_golden_values():
    for n, tau, k in _golden_keep_counts():
        assert oracle.keep_count(n, float(tau)) == k


def test_keep_count_equals_exact_rational_ceiling():
    for tau in ("0.004", "0.02", "0.03", "0.05", "0.07", "0.10", "0.15", "0.2", "0.25", "0.35", "0.5",
                "0.55", "0.7", "1.0"):
        fr = Fraction(tau)
        for n in list(range(1, 3000)) + list(range(3000, 20001, 7)) + [16384, 20000]:
            assert oracle.keep_count(n, float(tau)) == math.ceil(fr * n), (tau, n)
    assert oracle.keep_count(100, 0.0) == 0 and oracle.keep_count(0, 0.5) == 0
    assert oracle.keep_count(10, 1.0) == 10
