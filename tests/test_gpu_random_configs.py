"""Seeded random configurations of the three stages against the oracle: batch, heads, block count, ragged tail, head
dimension, storage type, uniform or per-row budgets, local cube forced or not, with or without a work order are drawn
together, so that combinations no hand-written case names get exercised.  Same bars as the other parity tests: scores at
the fp32 bound, selection bit-exact on the GPU's own scores, attention at the bound of its input type."""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import usv_oracle as orc
from paper_2512_05754_amd import synth

pytestmark = pytest.mark.gpu


def draw(seed):
    rng = np.random.default_rng([20251205, seed])
    nb = int(rng.choice([1, 2, 3, 5, 8, 13, 21, 34]))
    tail = int(rng.integers(1, 65))
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    ragged = nb > 1 and rng.random() < 0.5
    kmax = int(rng.integers(1, min(nb, 12) + 1))
    w = synth.Workload(f"rand{seed}", int(rng.integers(1, 3)), int(rng.integers(1, 4)), (nb - 1) * 64 + tail,
                       int(rng.choice([64, 128])), dtype, float(rng.choice([0.0, 1.0, 2.0])), 0 if ragged else kmax,
                       0 if not ragged else 0, 0 if not ragged else kmax, seed=9000 + seed)
    return w, ragged, kmax, bool(rng.random() < 0.3), bool(rng.random() < 0.5), rng


@pytest.mark.parametrize("seed", range(32))
def test_random_configuration(usv, seed):
    w, ragged, kmax, force_local, ordered, rng = draw(seed)
    Q, K, V = synth.gen_qkv(w)
    q, k, v = gu.up(Q), gu.up(K), gu.up(V)
    Qf, Kf, Vf = (synth.as_f32(x) for x in (Q, K, V))
    budgets = rng.integers(-1, kmax + 2, size=(w.batch, w.heads, w.nb)).astype(np.int32) if ragged else None
    what = f"{w.name}: B{w.batch} H{w.heads} Nv{w.seq_valid} d{w.head_dim} {w.dtype} kmax{kmax} ragged={ragged} local={force_local} ordered={ordered}"
    S = usv.block_scores(q, k, seq_valid=w.seq_valid)
    S_h = gu.down(S)
    gu.assert_f32_close(S_h, orc.block_scores(Qf, Kf, w.seq_valid), what + " scores")
    idx, cnt = usv.select_topk(S, k=0 if ragged else kmax, seq_valid=w.seq_valid, kmax=kmax,
                               budgets=None if budgets is None else gu.up(budgets), force_local=force_local)
    ridx, rcnt = orc.select_topk(S_h, kmax, w.seq_valid, budgets=budgets, kmax=kmax, force_local=force_local)
    assert np.array_equal(gu.down(idx), ridx) and np.array_equal(gu.down(cnt), rcnt), what + " selection"
    wo = usv.attn_work_order(cnt, kmax, idx=idx) if ordered else None
    out, lse = usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, return_lse=True, out_dtype=torch.float32,
                                     work_order=wo)
    O, L = orc.block_sparse_attn(Qf, Kf, Vf, ridx, rcnt, w.seq_valid)
    gu.assert_attn_close(gu.down(out), O, w.dtype, what)
    lse_h = gu.down(lse)
    live = np.isfinite(L)
    assert np.array_equal(np.isneginf(lse_h), ~live), what + " lse of rows without keys"
    if live.any():
        assert np.abs(lse_h[live] - L[live]).max() <= (1e-4 if w.dtype == "f32" else 2e-2), what + " lse"
    if w.dtype == "bf16":  # stored in the input type: round-to-nearest-even of the fp32-stored result, bit for bit
        out16 = usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, work_order=wo)
        gu.assert_bf16_store_is_rne(out16, out, what)


CUBES = [(4, 4, 4), (2, 4, 8), (1, 8, 8), (4, 2, 8), (8, 8, 1), (2, 2, 16)]


@pytest.mark.parametrize("seed", range(12))
def test_random_grid_in_the_cube_faithful_layout(usv, seed):
    """Random latent grids and cube shapes, one block per cube (cut cubes padded): the raster entry points with per-block
    valid counts against the oracle on the gathered tensors."""
    from test_gpu_cubes import faithful_case

    rng = np.random.default_rng([20251206, seed])
    cube = CUBES[int(rng.integers(len(CUBES)))]
    grid = tuple(int(rng.integers(1, 3 * c + 2)) for c in cube)
    blocks = int(np.prod([-(-g // c) for g, c in zip(grid, cube)]))
    keep = int(rng.integers(1, min(blocks, 9) + 1))
    B, Hh, d = int(rng.integers(1, 3)), int(rng.integers(1, 3)), int(rng.choice([64, 128]))
    what = f"grid {grid} cube {cube} B{B} H{Hh} d{d} keep {keep} of {blocks}"
    c = faithful_case(usv, grid, cube, B, Hh, d, keep, seed=8000 + seed)
    N, Nv = c["N"], c["Nv"]
    assert N == blocks * 64
    gu.assert_f32_close(gu.down(c["S"]), orc.block_scores(c["Qc"], c["Kc"], N, block_valid=c["o_valid"]), what + " scores")
    ridx, rcnt = orc.select_topk(gu.down(c["S"]), keep, N)
    assert np.array_equal(gu.down(c["idx"]), ridx) and np.array_equal(gu.down(c["cnt"]), rcnt), what
    O_ref, L_ref = orc.block_sparse_attn(c["Qc"], c["Kc"], c["Vc"], ridx, rcnt, N, block_valid=c["o_valid"])
    gu.assert_attn_close(gu.down(c["out"]), orc.order_scatter(O_ref, c["o_ord"], Nv), "bf16", what)
    want_lse = orc.order_scatter(L_ref[..., None], c["o_ord"], Nv)[..., 0]
    assert np.abs(gu.down(c["lse"]) - want_lse).max() <= 2e-2, what
