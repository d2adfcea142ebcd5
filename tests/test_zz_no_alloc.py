"""usv_block_scores_static (stage 1 with its pooled means in the library's static device array, for callers
that cannot allocate) against usv_block_scores: same kernels, so the scores must agree bit for bit, on two
calls in a row of which the second is smaller (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import usv_oracle as orc
from paper_2512_05754_amd import binding, synth

pytestmark = pytest.mark.gpu


def scores_both_ways(usv, w):
    Q, K, _ = synth.gen_qkv(w)
    q, k = gu.up(Q), gu.up(K)
    ref = usv.block_scores(q, k, seq_valid=w.seq_valid)
    out = torch.full_like(ref, float("nan"))
    before = torch.cuda.memory_allocated()
    got = usv.block_scores_static(q, k, out, seq_valid=w.seq_valid)
    assert torch.cuda.memory_allocated() == before  # nothing came from torch's allocator either
    torch.cuda.synchronize()
    assert got.data_ptr() == out.data_ptr()
    assert torch.equal(got.view(torch.int32), ref.view(torch.int32)), w.name
    return Q, K, got


def test_static_scratch_entry_point_matches_block_scores(usv):
    big = synth.Workload("static_big", 2, 3, 37 * 64 - 11, 128, "bf16", 2.0, 4, seed=901)
    small = synth.Workload("static_small", 1, 2, 5 * 64 - 30, 64, "f32", 2.0, 2, seed=902)
    for w in (big, small, big):  # the second call is the smaller one; then the large one again
        Q, K, got = scores_both_ways(usv, w)
        gu.assert_f32_close(gu.down(got), orc.block_scores(synth.as_f32(Q), synth.as_f32(K), w.seq_valid), w.name)


def test_static_scratch_entry_point_rejects_oversized_shapes(usv):
    limit = 64 << 20
    # 2 * B * Hh * nb * d * 4 bytes of pooled means: just over the limit
    B, Hh, nb, d = 2, 33, 1024, 128
    assert 2 * B * Hh * nb * d * 4 > limit
    q = torch.empty((1, 1, 64, d), dtype=torch.bfloat16, device=gu.DEV)
    sh = binding.UsvShape(B, Hh, nb * 64, nb * 64, d, 64, binding.USV_BF16)
    import ctypes

    L = usv.lib()
    rc = L.usv_block_scores_static(q.data_ptr(), q.data_ptr(), ctypes.byref(sh), q.data_ptr(), None)
    assert L.usv_status_string(rc).decode() == "USV_ERR_WORKSPACE"
    assert b"static scratch" in L.usv_last_error()
