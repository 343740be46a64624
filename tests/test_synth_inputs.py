"""The synthetic input generator: determinism, shapes, the drifting fixation, and the
planted-fixation ground truth seen through the oracle (CPU only)."""
import numpy as np
import torch

import fastocr_synth as fs
import oracle
from util import f32_to_bf16_bits


def test_config_shapes_follow_the_benchmark_configs():
    c1, c2, c3, c4, c5 = (fs.config(i) for i in range(1, 6))
    assert (c1.dtype, c1.n_q_heads, c1.n_kv_heads, c1.head_dim) == ("f32", 4, 1, 64)
    assert (c2.n_q_heads, c2.n_kv_heads, c2.head_dim, c2.steps, c2.warmup) == (28, 4, 128, 512, 4)
    assert c3.n_layers == 28 and c3.focal_layers == (2, 14) and c3.batch == 8
    assert (c4.batch, c4.n_q_heads, c4.n_kv_heads, c4.n_visual[0], c4.line_jump) == (16, 64, 8, 16384, 128)
    assert c5.paged and c5.batch == 32
    b1 = fs.make_batch(c1)
    assert b1.seq_len(1) == [288] and b1.n_vis == [256] and b1.vis_start == [15]
    assert oracle.keep_count(b1.n_vis[0], c1.taus[0]) == 13


def test_generation_is_chunk_independent_and_seeded():
    wl = fs.config(2, steps=3, n_visual=(256, 256), grid_w=(16, 16))
    a = fs.make_batch(wl, chunk_tokens=8192)
    b = fs.make_batch(wl, chunk_tokens=37)
    assert torch.equal(a.k, b.k) and torch.equal(a.v, b.v)
    c = fs.make_batch(wl, seed=fs.BASE_SEED + 1)
    assert not torch.equal(a.k, c.k)
    l1 = fs.make_batch(wl, layer=1)
    assert not torch.equal(a.k, l1.k)
    x = a.k.float()
    assert abs(x.mean().item()) < 0.02 and abs(x.std().item() - 1.0) < 0.02
    assert abs((a.k.float() * a.v.float()).mean().item()) < 0.02       # K and V independent


def test_bf16_bits_reach_the_oracle_unchanged():
    x = torch.randn(1000, dtype=torch.float32)
    bits = fs.to_oracle_array(x.to(torch.bfloat16))
    assert bits.dtype == np.uint16 and np.array_equal(bits, f32_to_bf16_bits(x.numpy()))


def test_ragged_paged_batch_geometry():
    wl = fs.config(5, batch=6, steps=4, n_visual=(128, 1024), grid_w=(8, 32), text_prefix=(3, 40),
                   page_tokens=16)
    bt = fs.make_batch(wl)
    assert len(set(bt.n_vis)) > 1 and all(128 - 32 <= n <= 1024 for n in bt.n_vis)
    assert all(n == w * h for n, w, h in zip(bt.n_vis, bt.grid_w, bt.grid_h))
    table = bt.block_table.cpu().numpy()
    used = []
    for b in range(wl.batch):
        cap = bt.n_vis[b] + bt.prefix[b] + wl.steps
        used += table[b, : -(-cap // 16)].tolist()
    assert len(used) == len(set(used)) == bt.k.shape[0]                   # every page owned exactly once
    # the same rows come back through the block table as from a contiguous batch
    flat = fs.make_batch(fs.config(5, batch=6, steps=4, n_visual=(128, 1024), grid_w=(8, 32),
                                   text_prefix=(3, 40), page_tokens=16, paged=False))
    toks = torch.tensor([0, 5, 17, 100])
    for b in (0, 3):
        assert torch.equal(bt.rows("k", b, toks), flat.rows("k", b, toks))
        assert torch.equal(bt.rows("v", b, toks), flat.rows("v", b, toks))


def test_centre_drifts_in_raster_order_with_line_jumps():
    wl = fs.config(4, batch=2, steps=300, n_visual=(1024, 1024), grid_w=(32, 32), line_jump=128)
    bt = fs.make_batch(fs.config(4, batch=2, steps=1, n_visual=(1024, 1024), grid_w=(32, 32)))
    bt.wl = wl
    cs = fs.centres(bt)
    for seq in cs:
        assert len(seq) == 300 and 0 <= seq[0] < 32
        for t in range(1, 300):
            if t % 128 == 0:
                assert seq[t] % 32 == 0                                    # start of a row
            else:
                assert (seq[t] - seq[t - 1]) % 1024 in (1, 2)
    assert cs[0] != cs[1]


def test_window_is_clipped_not_wrapped():
    assert fs.window_cells(0, 16, 16, 1) == [0, 1, 16, 17]
    assert fs.window_cells(15, 16, 16, 1) == [14, 15, 30, 31]
    assert len(fs.window_cells(8 * 16 + 8, 16, 16, 2)) == 25
    assert fs.window_cells(255, 16, 16, 1) == [238, 239, 254, 255]


def test_query_is_window_mean_plus_small_noise():
    wl = fs.config(1)
    bt = fs.make_batch(wl)
    c = fs.centres(bt)[0][0]
    q = fs.queries_for_step(bt, 1, [c]).double()
    cells = torch.tensor(fs.window_cells(c, 16, 16, 1)) + bt.vis_start[0]
    mean = bt.k[0, 0, cells].double().mean(0)
    resid = q[0] - mean                                                     # [Hq, d], sigma = 0.1
    assert 0.07 < resid.std().item() < 0.13
    assert not torch.equal(q[0, 0], q[0, 1])                                # noise differs per head


def _recall(wl, seed):
    bt = fs.make_batch(wl, seed=seed)
    c = fs.centres(bt)[0][0]
    q = fs.queries_for_step(bt, 1, [c])
    cache = oracle.Cache.from_bhsd(fs.to_oracle_array(bt.k), fs.to_oracle_array(bt.v))
    scale = float(np.float32(wl.head_dim ** -0.5))
    sc, _, _ = oracle.focal_score(cache, bt.seq_len(1), bt.vis_start, bt.n_vis, fs.to_oracle_array(q), scale)
    k = oracle.keep_count(bt.n_vis[0], wl.taus[0])
    sel = set(oracle.topk(sc[0], k).tolist())
    win = fs.window_cells(c, bt.grid_w[0], bt.grid_h[0], wl.window_r)
    return len(sel & set(win)) / len(win), k / bt.n_vis[0]


def test_planted_fixation_is_found_by_the_oracle_statistically():
    # The window keys have the highest expected logit but the background's order statistics
    # compete, so recall is high, not certain; chance level is tau = 5 %.
    rec = [_recall(fs.config(1), fs.BASE_SEED + 17 * s)[0] for s in range(30)]
    assert np.mean(rec) > 0.6 and min(rec) >= 0.3
    wl = fs.config(2, steps=1)
    rec2 = [_recall(wl, fs.BASE_SEED + 5 * s)[0] for s in range(3)]
    assert np.mean(rec2) > 0.7


def test_plain_fill_keeps_geometry_tables_and_distribution():
    """The fill used under hardware counters: one random-normal launch per tensor instead of the seeded
    generator's many; everything but the values is the seeded batch's."""
    wl = fs.config(5, batch=3, n_visual=(300, 700), steps=8)
    a = fs.make_batch(wl, device="cpu", plain_fill=True)
    b = fs.make_batch(wl, device="cpu")
    assert (a.n_vis, a.prefix, a.vis_start, a.grid_w, a.grid_h, a.cap) == (b.n_vis, b.prefix, b.vis_start, b.grid_w, b.grid_h, b.cap)
    assert torch.equal(a.block_table, b.block_table)
    assert a.k.shape == b.k.shape and a.v.shape == b.v.shape and a.k.dtype == b.k.dtype
    for x in (a.k, a.v):
        x = x.float()
        assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1.0) < 0.02
    assert not torch.equal(a.k, a.v)
