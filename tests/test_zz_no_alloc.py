"""The entry point that allocates nothing (fastocr_dense_decode_attn_static: split partials in the
library's static device buffer) against fastocr_dense_decode_attn with a caller-provided workspace:
bit-identical outputs (the kernels are the same), and both within the oracle's bar, on calls in a
row that share the buffer -- the second and third on smaller inputs, so stale partials of a larger
call lie behind theirs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_17447_amd as fo
from paper_2605_17447_amd import binding as fb
from util import TinyCase

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import DEV, check_out, problem_from_case


def _both(p, what):
    ref, ref_lse = oracle.decode_attn(*p.oracle_args())
    want, want_lse = p.dense(want_lse=True)
    out = torch.full_like(p.q, 3.0)
    lse = torch.zeros((p.B, p.Hq), dtype=torch.float32, device=DEV)
    before = torch.cuda.memory_allocated()
    fo.dense_decode_attn_static(p.cache, p.batch, p.q, p.scale, out, lse)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert torch.equal(out, want), what + ": output differs from the workspace entry point"
    assert torch.equal(lse, want_lse), what + ": lse differs from the workspace entry point"
    check_out(out, ref, what + " vs oracle")
    nz = [b for b in range(p.B) if p.seq_len[b] > 0]
    assert np.allclose(lse.cpu().numpy()[nz], ref_lse[nz], rtol=2e-5, atol=2e-5), what + " lse vs oracle"


def test_static_scratch_entry_point_matches_the_workspace_one():
    big = TinyCase(seed=71, B=4, Hq=28, Hkv=4, d=128, n_vis=[3000, 1777, 2500, 64], pre=[32, 5, 0, 3],
                   post=[41, 130, 7, 0], dtype="bf16")
    small = TinyCase(seed=72, B=2, Hq=28, Hkv=4, d=128, n_vis=[500, 300], pre=[3, 9], post=[20, 1], dtype="bf16")
    plain = TinyCase(seed=73, B=2, Hq=4, Hkv=2, d=64, n_vis=[150, 99], pre=[8, 3], post=[5, 7], dtype="f32")
    _both(problem_from_case(big), "first call")
    _both(problem_from_case(small), "second call, smaller input")
    _both(problem_from_case(plain), "third call, fp32 plain-FMA kernels")
    _both(problem_from_case(big), "fourth call, the large input again")


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    # 2000 sequences x 64 query heads x 2 ranges x 130 floats: about 130 MB of partials
    B = 2000
    k = torch.zeros((B, 8, 64, 128), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((B, 64, 128), dtype=torch.bfloat16, device=DEV)
    cache = fo.KvCache(k, k)
    batch = fo.SeqBatch.from_lists([64] * B, [0] * B, [32] * B, DEV)
    assert fo.workspace_bytes(fb.OP_DENSE_DECODE_ATTN, cache, batch, 64) > fb.STATIC_SCRATCH_BYTES
    with pytest.raises(fo.FastOcrError) as e:
        fo.dense_decode_attn_static(cache, batch, q, 0.1, torch.zeros_like(q))
    assert e.value.status == fb.ETOOLARGE
