"""GPU parity of the raster-order entry points: the three stages on raster tensors must give what
usv_cube_gather -> stage -> usv_cube_scatter gives (bit for bit: same arithmetic, only the addresses
differ), and that in turn is checked against the oracle."""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import usv_oracle as orc
from paper_2512_05754_amd import synth

pytestmark = pytest.mark.gpu


def raster_inputs(w, grid, cube):
    Qc, Kc, Vc = synth.gen_qkv(w)  # cube-major with the block structure; the raster tensors are their scatter
    return tuple(orc.cube_scatter(x, grid, cube) for x in (Qc, Kc, Vc))


CASES = [
    ((5, 8, 12), (4, 4, 4), 1, 2, 128, 3),     # 480 tokens, cut cubes, ragged tail
    ((4, 8, 8), (4, 4, 4), 2, 3, 128, 2),      # divisible grid, two batch elements
    ((7, 9, 10), (4, 4, 4), 1, 2, 64, 4),      # d = 64
    ((3, 12, 70), (1, 8, 8), 1, 1, 128, 30),   # flat cubes, lists longer than the request look-ahead
    ((6, 20, 40), (4, 4, 4), 1, 1, 128, 70),   # lists longer than 64 entries (index reload)
]


@pytest.mark.parametrize("grid,cube,B,Hh,d,keep", CASES, ids=lambda v: str(v).replace(" ", ""))
def test_raster_path_equals_gather_path_and_oracle(usv, grid, cube, B, Hh, d, keep):
    Nv = grid[0] * grid[1] * grid[2]
    w = synth.Workload("raster", B, Hh, Nv, d, "bf16", 2.0, keep, seed=81 + d + keep)
    Qr, Kr, Vr = raster_inputs(w, grid, cube)
    q, k, v = gu.up(Qr), gu.up(Kr), gu.up(Vr)
    N = w.seq_len
    order = usv.cube_order(grid, cube, seq_len=N)
    np.testing.assert_array_equal(order.cpu().numpy()[:Nv], orc.cube_token_order(grid, cube))
    assert not order.cpu().numpy()[Nv:].any()
    # reference path on the GPU: gather, three stages, scatter
    qc, kc, vc = (usv.cube_gather(x, grid, cube, seq_len=N) for x in (q, k, v))
    S_ref = usv.block_scores(qc, kc, seq_valid=Nv)
    S = usv.block_scores_raster(q, k, order)
    assert torch.equal(S, S_ref)
    idx, cnt = usv.select_topk(S, k=keep, seq_valid=Nv)
    for odt in (torch.float32, torch.bfloat16):
        o_ref, lse_ref = usv.block_sparse_attn(qc, kc, vc, idx, cnt, seq_valid=Nv, out_dtype=odt, return_lse=True)
        o_ref_r = usv.cube_scatter(o_ref, grid, cube)
        out, lse = usv.block_sparse_attn_raster(q, k, v, order, idx, cnt, out_dtype=odt, return_lse=True)
        assert torch.equal(out.view(torch.int32 if odt == torch.float32 else torch.int16),
                           o_ref_r.view(torch.int32 if odt == torch.float32 else torch.int16))
        lse_r = gu.down(lse_ref)[:, :, :Nv][:, :, np.argsort(orc.cube_token_order(grid, cube))]
        np.testing.assert_array_equal(gu.down(lse), lse_r)
    # and against the oracle
    Qf, Kf, Vf = (orc.cube_gather(synth.as_f32(x), grid, cube, N) for x in (Qr, Kr, Vr))
    ridx, rcnt = orc.select_topk(gu.down(S), keep, Nv)
    np.testing.assert_array_equal(idx.cpu().numpy(), ridx)
    ref = orc.cube_scatter(orc.block_sparse_attn(Qf, Kf, Vf, ridx, rcnt, Nv)[0], grid, cube)
    out = usv.block_sparse_attn_raster(q, k, v, order, idx, cnt, out_dtype=torch.float32)
    gu.assert_attn_close(gu.down(out), ref, "bf16", "raster attention")


def test_raster_path_on_projection_layout(usv):
    """Q, K, V as one projection output [B, Nv, 3, Hh, d] (strided views) and the output written as [B, Nv, Hh*d]."""
    grid, cube, B, Hh, d, keep = (5, 8, 12), (4, 4, 4), 2, 3, 128, 3
    Nv = 480
    w = synth.Workload("raster_proj", B, Hh, Nv, d, "bf16", 2.0, keep, seed=91)
    Qr, Kr, Vr = raster_inputs(w, grid, cube)
    qkv = torch.stack([gu.up(x) for x in (Qr, Kr, Vr)], dim=0)          # [3, B, Hh, Nv, d]
    packed = qkv.permute(1, 3, 0, 2, 4).contiguous()                     # [B, Nv, 3, Hh, d]
    q, k, v = (packed[:, :, t].permute(0, 2, 1, 3) for t in range(3))    # [B, Hh, Nv, d] views, token stride 3*Hh*d
    order = usv.cube_order(grid, cube)
    S = usv.block_scores_raster(q, k, order)
    idx, cnt = usv.select_topk(S, k=keep, seq_valid=Nv)
    buf = torch.zeros((B, Nv, Hh, d), dtype=torch.bfloat16, device=gu.DEV)
    usv.block_sparse_attn_raster(q, k, v, order, idx, cnt, out=buf.permute(0, 2, 1, 3))
    ref = usv.block_sparse_attn_raster(gu.up(Qr), gu.up(Kr), gu.up(Vr), order, idx, cnt)
    assert torch.equal(buf.permute(0, 2, 1, 3).contiguous().view(torch.int16), ref.view(torch.int16))
    assert torch.equal(S, usv.block_scores_raster(gu.up(Qr), gu.up(Kr), order))


def test_raster_path_full_size_480p(usv):
    """The 480p latent grid with all 12 heads: raster path against the gather path, bit for bit."""
    grid, cube = (21, 30, 52), (4, 4, 4)
    w = synth.WAN13_480P
    Qr, Kr, Vr = raster_inputs(w, grid, cube)
    q, k, v = gu.up(Qr), gu.up(Kr), gu.up(Vr)
    order = usv.cube_order(grid, cube)
    S = usv.block_scores_raster(q, k, order)
    idx, cnt = usv.select_topk(S, k=w.keep, seq_valid=w.seq_valid)
    out = usv.block_sparse_attn_raster(q, k, v, order, idx, cnt, out_dtype=torch.float32)
    qc, kc, vc = (usv.cube_gather(x, grid, cube) for x in (q, k, v))
    assert torch.equal(S, usv.block_scores(qc, kc, seq_valid=w.seq_valid))
    o_ref = usv.cube_scatter(usv.block_sparse_attn(qc, kc, vc, idx, cnt, seq_valid=w.seq_valid, out_dtype=torch.float32),
                             grid, cube)
    assert torch.equal(out.view(torch.int32), o_ref.view(torch.int32))
    # ... and the raster-order output against the oracle itself: sampled (head, query cube) rows, the oracle working
    # on cube-major copies it gathers on its own and answering at the raster positions of the cube's tokens
    Qc, Kc, Vc = synth.gen_qkv(w)  # raster_inputs() scatters exactly these
    idx_h, cnt_h, out_h = gu.down(idx), gu.down(cnt), out.cpu().numpy()
    ridx, rcnt = orc.select_topk(gu.down(S)[:, :2], w.keep, w.seq_valid)
    assert np.array_equal(idx_h[:, :2], ridx) and np.array_equal(cnt_h[:, :2], rcnt)
    tok = orc.cube_token_order(grid, cube)  # raster index of cube-major position p
    rng = np.random.default_rng(7)
    worst = 0.0
    for h in rng.choice(w.heads, size=4, replace=False):
        blocks = sorted(set(rng.choice(w.nb, size=16, replace=False).tolist()) | {w.nb - 1})
        ref = gu.oracle_attn_blocks(Qc[0, h], Kc[0, h], Vc[0, h], idx_h[0, h], cnt_h[0, h], w.seq_valid, blocks)
        for i in blocks:
            nvalid = min(64, w.seq_valid - 64 * i)
            got = out_h[0, h, tok[64 * i:64 * i + nvalid]]
            mx, _ = gu.assert_attn_close(got, ref[i][0][:nvalid], "bf16", f"raster 480p head {h} cube {i}")
            worst = max(worst, mx)
    print(f"\nraster 480p against the oracle: max|err| {worst:.3e} on 4 x 17 sampled cubes")


@pytest.mark.parametrize("grid,cube,B,Hh,d,keep", [CASES[0], CASES[1], CASES[2]], ids=lambda v: str(v).replace(" ", ""))
def test_raster_second_branch_equals_gather_path(usv, grid, cube, B, Hh, d, keep):
    """usv_coarse_attn_raster and usv_block_sparse_attn_raster_fused (own cube forced, raster-order gates) against
    gather -> usv_coarse_attn / usv_block_sparse_attn_fused -> scatter: bit for bit."""
    Nv = grid[0] * grid[1] * grid[2]
    w = synth.Workload("raster2", B, Hh, Nv, d, "bf16", 2.0, keep, seed=171 + d + keep)
    Qr, Kr, Vr = raster_inputs(w, grid, cube)
    q, k, v = gu.up(Qr), gu.up(Kr), gu.up(Vr)
    N = w.seq_len
    gen = torch.Generator(device=gu.DEV).manual_seed(5)
    gates = [torch.rand((B, Hh, Nv, d), device=gu.DEV, generator=gen).to(torch.bfloat16) for _ in range(2)]
    order = usv.cube_order(grid, cube, seq_len=N)
    S = usv.block_scores_raster(q, k, order)
    idx, cnt = usv.select_topk(S, k=keep, seq_valid=Nv, force_local=True)
    coarse = usv.coarse_attn_raster(S, v, order)
    qc, kc, vc, g0, g1 = (usv.cube_gather(x, grid, cube, seq_len=N) for x in (q, k, v, gates[0], gates[1]))
    coarse_ref = usv.coarse_attn(S, vc, seq_valid=Nv)
    assert torch.equal(coarse.view(torch.int32), coarse_ref.view(torch.int32))
    for odt in (torch.float32, torch.bfloat16):
        for gf, gc, rf, rc in ((gates[0], gates[1], g0, g1), (None, gates[1], None, g1), (None, None, None, None)):
            out = usv.block_sparse_attn_raster(q, k, v, order, idx, cnt, out_dtype=odt, coarse=coarse, gate_fine=gf,
                                               gate_coarse=gc)
            ref = usv.cube_scatter(usv.block_sparse_attn(qc, kc, vc, idx, cnt, seq_valid=Nv, out_dtype=odt, coarse=coarse_ref,
                                                         gate_fine=rf, gate_coarse=rc), grid, cube)
            it = torch.int32 if odt == torch.float32 else torch.int16
            assert torch.equal(out.view(it), ref.view(it))
    # and the fused result against the oracle's two branches
    Qf, Kf, Vf = (orc.cube_gather(synth.as_f32(x), grid, cube, N) for x in (Qr, Kr, Vr))
    fine = orc.block_sparse_attn(Qf, Kf, Vf, gu.down(idx), gu.down(cnt), Nv)[0]
    co = orc.coarse_attn(gu.down(S), Vf, Nv)
    gcm = [orc.cube_gather(gu.down(g).astype(np.float64), grid, cube, N) for g in gates]
    want = orc.cube_scatter(orc.fuse_outputs(fine, co, Nv, gcm[0], gcm[1]), grid, cube)
    got = usv.block_sparse_attn_raster(q, k, v, order, idx, cnt, out_dtype=torch.float32, coarse=coarse,
                                       gate_fine=gates[0], gate_coarse=gates[1])
    gu.assert_attn_close(gu.down(got), want, "bf16", "raster fused attention")


def test_raster_every_list_length(usv):
    """Every list length from 0 to 20 on raster tensors (the order ring and the K/V ring of the raster kernel run
    through all their phases and partial last rounds), against the gather path bit for bit."""
    grid, cube, B, Hh, d, kmax = (8, 12, 20), (4, 4, 4), 1, 2, 128, 20
    Nv = grid[0] * grid[1] * grid[2]
    w = synth.Workload("raster_lengths", B, Hh, Nv, d, "bf16", 2.0, kmax, seed=411)
    Qr, Kr, Vr = raster_inputs(w, grid, cube)
    q, k, v = gu.up(Qr), gu.up(Kr), gu.up(Vr)
    N, nb = w.seq_len, w.nb
    rng = np.random.default_rng(8)
    idx = np.full((B, Hh, nb, kmax), -1, dtype=np.int32)
    cnt = np.zeros((B, Hh, nb), dtype=np.int32)
    for h in range(Hh):
        for i in range(nb):
            c = (i + 5 * h) % (kmax + 1)
            idx[0, h, i, :c] = np.sort(rng.choice(nb, size=c, replace=False))
            cnt[0, h, i] = c
    order = usv.cube_order(grid, cube, seq_len=N)
    qc, kc, vc = (usv.cube_gather(x, grid, cube, seq_len=N) for x in (q, k, v))
    ref = usv.cube_scatter(usv.block_sparse_attn(qc, kc, vc, gu.up(idx), gu.up(cnt), seq_valid=Nv, out_dtype=torch.float32),
                           grid, cube)
    out = usv.block_sparse_attn_raster(q, k, v, order, gu.up(idx), gu.up(cnt), out_dtype=torch.float32)
    assert torch.equal(out.view(torch.int32), ref.view(torch.int32))
