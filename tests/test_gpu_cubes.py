"""GPU parity of the cube-faithful mode: one cube per block, the cubes that the grid boundary cuts padded to a block
of their own (usv_cube_order_padded + view->block_valid on the raster entry points), against the oracle's
cube_token_order_padded and its per-block valid counts."""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import usv_oracle as orc
from paper_2512_05754_amd import synth

pytestmark = pytest.mark.gpu

GRIDS = [((5, 6, 7), (4, 4, 4)), ((21, 30, 52), (4, 4, 4)), ((4, 8, 8), (4, 4, 4)), ((3, 12, 70), (1, 8, 8)),
         ((1, 1, 1), (4, 4, 4))]


@pytest.mark.parametrize("grid,cube", GRIDS, ids=lambda v: str(v).replace(" ", ""))
def test_padded_order_table_matches_oracle(usv, grid, cube):
    order, valid = usv.cube_order_padded(grid, cube)
    ref_order, ref_valid = orc.cube_token_order_padded(grid, cube)
    got = order.cpu().numpy()
    np.testing.assert_array_equal(valid.cpu().numpy(), ref_valid)
    np.testing.assert_array_equal(got[ref_order >= 0], ref_order[ref_order >= 0])
    assert not got[ref_order < 0].any()  # padding positions hold a readable index: 0


def faithful_case(usv, grid, cube, B, Hh, d, keep, seed, out_dtype=torch.float32):
    Nv = grid[0] * grid[1] * grid[2]
    w = synth.Workload("cubes", B, Hh, Nv, d, "bf16", 2.0, keep, seed=seed)
    Qr, Kr, Vr = synth.gen_raster_qkv(w, grid, cube)
    q, k, v = gu.up(Qr), gu.up(Kr), gu.up(Vr)
    order, bv = usv.cube_order_padded(grid, cube)
    N = order.numel()
    S = usv.block_scores_raster(q, k, order, block_valid=bv)
    idx, cnt = usv.select_topk(S, k=keep)  # every block is a candidate: seq_valid = seq_len
    out, lse = usv.block_sparse_attn_raster(q, k, v, order, idx, cnt, out_dtype=out_dtype, return_lse=True, block_valid=bv)
    torch.cuda.synchronize()
    o_ord, o_valid = orc.cube_token_order_padded(grid, cube)
    Qc, Kc, Vc = (orc.order_gather(synth.as_f32(x), o_ord) for x in (Qr, Kr, Vr))
    return dict(w=w, N=N, Nv=Nv, S=S, idx=idx, cnt=cnt, out=out, lse=lse, order=order, bv=bv, q=q, k=k, v=v,
                o_ord=o_ord, o_valid=o_valid, Qc=Qc, Kc=Kc, Vc=Vc, raw=(Qr, Kr, Vr))


CASES = [
    ((5, 6, 7), (4, 4, 4), 1, 2, 128, 3),      # every cube but one is cut
    ((7, 9, 10), (4, 4, 4), 2, 2, 64, 4),      # d = 64, two batch elements
    ((3, 12, 70), (1, 8, 8), 1, 1, 128, 9),    # flat cubes
    ((6, 20, 41), (4, 4, 4), 1, 1, 128, 70),   # lists longer than 64 entries (the ids and their counts are reloaded)
    ((8, 8, 8), (4, 4, 4), 1, 2, 128, 3),      # nothing cut: the mode changes nothing
]


@pytest.mark.parametrize("grid,cube,B,Hh,d,keep", CASES, ids=lambda v: str(v).replace(" ", ""))
def test_cube_faithful_stages_against_oracle(usv, grid, cube, B, Hh, d, keep):
    c = faithful_case(usv, grid, cube, B, Hh, d, keep, seed=600 + d + keep)
    N, Nv = c["N"], c["Nv"]
    S_ref = orc.block_scores(c["Qc"], c["Kc"], N, block_valid=c["o_valid"])
    gu.assert_f32_close(gu.down(c["S"]), S_ref, "scores")
    ridx, rcnt = orc.select_topk(gu.down(c["S"]), keep, N)
    assert np.array_equal(gu.down(c["idx"]), ridx) and np.array_equal(gu.down(c["cnt"]), rcnt)
    O_ref, L_ref = orc.block_sparse_attn(c["Qc"], c["Kc"], c["Vc"], ridx, rcnt, N, block_valid=c["o_valid"])
    want = orc.order_scatter(O_ref, c["o_ord"], Nv)
    gu.assert_attn_close(gu.down(c["out"]), want, "bf16", "cube-faithful attention")
    want_lse = orc.order_scatter(L_ref[..., None], c["o_ord"], Nv)[..., 0]
    assert np.isfinite(want_lse).all()
    assert np.abs(gu.down(c["lse"]) - want_lse).max() <= 2e-2
    # the bf16-stored output is the fp32-stored one rounded to nearest even
    out_bf = usv.block_sparse_attn_raster(c["q"], c["k"], c["v"], c["order"], c["idx"], c["cnt"], block_valid=c["bv"])
    gu.assert_bf16_store_is_rne(out_bf, c["out"], "cube-faithful")
    # a work order changes which workgroup takes which cube, not a bit of the result
    wo = usv.attn_work_order(c["cnt"], keep, idx=c["idx"])
    out_wo, lse_wo = usv.block_sparse_attn_raster(c["q"], c["k"], c["v"], c["order"], c["idx"], c["cnt"], out_dtype=torch.float32,
                                                  return_lse=True, block_valid=c["bv"], work_order=wo)
    assert torch.equal(out_wo.view(torch.int32), c["out"].view(torch.int32)) and torch.equal(lse_wo, c["lse"])
    if Nv == N:  # no cube is cut: bit for bit what the packed order gives
        order0 = usv.cube_order(grid, cube)
        assert torch.equal(order0, c["order"])
        ref = usv.block_sparse_attn_raster(c["q"], c["k"], c["v"], order0, c["idx"], c["cnt"], out_dtype=torch.float32)
        assert torch.equal(ref.view(torch.int32), c["out"].view(torch.int32))


def test_cube_faithful_second_branch(usv):
    """usv_coarse_attn_raster and the fused store with per-block valid counts, against the oracle's two branches."""
    grid, cube, B, Hh, d, keep = (5, 10, 9), (4, 4, 4), 1, 2, 128, 4
    c = faithful_case(usv, grid, cube, B, Hh, d, keep, seed=731)
    N, Nv = c["N"], c["Nv"]
    gen = torch.Generator(device=gu.DEV).manual_seed(9)
    gates = [torch.rand((B, Hh, Nv, d), device=gu.DEV, generator=gen).to(torch.bfloat16) for _ in range(2)]
    idx, cnt = usv.select_topk(c["S"], k=keep, force_local=True)
    coarse = usv.coarse_attn_raster(c["S"], c["v"], c["order"], block_valid=c["bv"])
    C_ref = orc.coarse_attn(gu.down(c["S"]), c["Vc"], N, block_valid=c["o_valid"])
    gu.assert_f32_close(gu.down(coarse), C_ref, "cube-level branch")
    got = usv.block_sparse_attn_raster(c["q"], c["k"], c["v"], c["order"], idx, cnt, out_dtype=torch.float32, coarse=coarse,
                                       gate_fine=gates[0], gate_coarse=gates[1], block_valid=c["bv"])
    fine = orc.block_sparse_attn(c["Qc"], c["Kc"], c["Vc"], gu.down(idx), gu.down(cnt), N, block_valid=c["o_valid"])[0]
    gcm = [orc.order_gather(gu.down(g).astype(np.float64), c["o_ord"]) for g in gates]
    want = orc.order_scatter(orc.fuse_outputs(fine, C_ref, N, gcm[0], gcm[1]), c["o_ord"], Nv)
    err = np.abs(gu.down(got) - want)
    assert (err <= gu.BF16_MAX_ABS).all(), err.max()  # gates in [0, 1): they do not amplify the attention error


def test_cube_faithful_full_size_480p(usv):
    """The 480p latent grid, 12 heads, one block per cube: 624 blocks (169 of them cut cubes of 8..32 tokens), keep 62."""
    grid, cube = (21, 30, 52), (4, 4, 4)
    keep = synth.keep_count(0.10, 624)
    c = faithful_case(usv, grid, cube, 1, 12, 128, keep, seed=20251206)
    N, Nv = c["N"], c["Nv"]
    assert N == 624 * 64 and keep == 62
    S_h, idx_h, cnt_h = gu.down(c["S"]), gu.down(c["idx"]), gu.down(c["cnt"])
    out_h, lse_h = c["out"].cpu().numpy(), c["lse"].cpu().numpy()
    assert np.isfinite(out_h).all() and np.isfinite(lse_h).all()
    rng = np.random.default_rng(5)
    cut = np.nonzero(c["o_valid"] < 64)[0]
    worst = 0.0
    for h in rng.choice(12, size=4, replace=False):
        ref_S = orc.block_scores(c["Qc"][:, h:h + 1], c["Kc"][:, h:h + 1], N, block_valid=c["o_valid"])
        gu.assert_f32_close(S_h[:, h:h + 1], ref_S, f"scores head {h}")
        ridx, rcnt = orc.select_topk(S_h[:, h:h + 1], keep, N)
        assert np.array_equal(idx_h[:, h:h + 1], ridx) and np.array_equal(cnt_h[:, h:h + 1], rcnt)
        blocks = sorted(set(rng.choice(624, size=10, replace=False).tolist()) | set(rng.choice(cut, size=6, replace=False).tolist()))
        O, L = orc.block_sparse_attn_head(c["Qc"][0, h], c["Kc"][0, h], c["Vc"][0, h], idx_h[0, h], cnt_h[0, h], N, None,
                                          blocks, block_valid=c["o_valid"])
        for i in blocks:
            n = c["o_valid"][i]
            tok = c["o_ord"][64 * i:64 * i + n]
            mx, _ = gu.assert_attn_close(out_h[0, h, tok], O[64 * i:64 * i + n], "bf16", f"head {h} cube {i}")
            worst = max(worst, mx)
            assert np.abs(lse_h[0, h, tok] - L[64 * i:64 * i + n]).max() <= 2e-2
    print(f"\ncube-faithful 480p: max|err| {worst:.3e} on 4 x 16 sampled cubes")
