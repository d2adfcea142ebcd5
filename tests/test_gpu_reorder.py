"""GPU parity of the raster <-> cube-major reorder against the oracle: byte work, so bit-exact.

Inputs are random bit patterns (every uint16 / uint32 value is a legal payload for a copy), compared
as integers so that NaN payloads cannot hide a difference."""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import usv_oracle as orc
from paper_2512_05754_amd import synth

pytestmark = pytest.mark.gpu

CASES = [
    # grid, cube, B, Hh, d, dtype
    ((8, 8, 8), (4, 4, 4), 1, 2, 64, "bf16"),      # divisible
    ((5, 6, 7), (4, 4, 4), 2, 3, 128, "bf16"),     # cut along every axis, ragged tail
    ((5, 6, 7), (4, 4, 4), 1, 2, 128, "f32"),
    ((1, 9, 9), (4, 4, 4), 1, 1, 64, "f32"),       # a single frame: every cube is cut
    ((3, 3, 3), (4, 4, 4), 1, 1, 64, "bf16"),      # grid smaller than one cube
    ((3, 17, 19), (1, 8, 8), 1, 2, 128, "bf16"),   # flat cubes
    ((5, 9, 20), (2, 4, 8), 2, 1, 64, "bf16"),
    ((21, 30, 52), (4, 4, 4), 1, 1, 128, "bf16"),  # the 480p latent grid, one head
]


def bits(rng, shape, dtype):
    if dtype == "bf16":
        return rng.integers(0, 1 << 16, size=shape, dtype=np.uint16)
    return rng.integers(0, 1 << 32, size=shape, dtype=np.uint32)


def to_dev(x):
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).to(gu.DEV).view(torch.bfloat16)
    return torch.from_numpy(x.view(np.int32)).to(gu.DEV).view(torch.float32)


def to_bits(t):
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().view(torch.int32).cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("grid,cube,B,Hh,d,dtype", CASES, ids=lambda v: str(v).replace(" ", ""))
def test_gather_and_scatter_match_oracle(usv, grid, cube, B, Hh, d, dtype):
    rng = np.random.default_rng([17, *grid, d])
    Nv = grid[0] * grid[1] * grid[2]
    N = -(-Nv // 64) * 64 + 64  # one whole block of padding on top of the ragged tail
    X = bits(rng, (B, Hh, Nv, d), dtype)
    ref = orc.cube_gather(X, grid, cube, N)
    out = to_dev(bits(rng, (B, Hh, N, d), dtype))  # pre-filled with garbage: padding must be overwritten
    got = usv.cube_gather(to_dev(X), grid, cube, seq_len=N, out=out)
    np.testing.assert_array_equal(to_bits(got), ref)
    # inverse, from a cube-major tensor with garbage in the padding rows
    Y = bits(rng, (B, Hh, N, d), dtype)
    back = usv.cube_scatter(to_dev(Y), grid, cube)
    np.testing.assert_array_equal(to_bits(back), orc.cube_scatter(Y, grid, cube))
    # and the round trip is the identity
    np.testing.assert_array_equal(to_bits(usv.cube_scatter(got, grid, cube)), X)


def test_projection_layout_via_strides(usv):
    """Raster tensor laid out [B, Nv, Hh*d] (what a QKV projection writes), passed as a strided view."""
    grid, cube, B, Hh, d = (5, 6, 7), (4, 4, 4), 2, 3, 64
    rng = np.random.default_rng(5)
    Nv, N = 210, 256
    X = bits(rng, (B, Nv, Hh, d), "bf16")
    xv = to_dev(X).permute(0, 2, 1, 3)  # [B, Hh, Nv, d] view, token stride Hh*d
    assert not xv.is_contiguous()
    got = usv.cube_gather(xv, grid, cube, seq_len=N)
    ref = orc.cube_gather(X.transpose(0, 2, 1, 3), grid, cube, N)
    np.testing.assert_array_equal(to_bits(got), ref)
    # scatter into the same layout; the buffer's other bytes must stay as they were
    Y = bits(rng, (B, Hh, N, d), "bf16")
    buf = torch.zeros((B, Nv, Hh, d), dtype=torch.bfloat16, device=gu.DEV)
    usv.cube_scatter(to_dev(Y), grid, cube, out=buf.permute(0, 2, 1, 3))
    np.testing.assert_array_equal(to_bits(buf).transpose(0, 2, 1, 3), orc.cube_scatter(Y, grid, cube))


def test_pipeline_from_raster_tokens(usv):
    """Raster Q/K/V -> gather -> scores -> top-k -> attention -> scatter, against the oracle doing the same."""
    grid, cube = (5, 8, 12), (4, 4, 4)  # 480 tokens: 4 whole cubes + cut ones, padded to 512
    w = synth.Workload("raster_pipe", 1, 2, 480, 128, "bf16", 2.0, 3, seed=21)
    Qc, Kc, Vc = synth.gen_qkv(w)  # generated in cube-major order; the raster tensors are their scatter
    Qr, Kr, Vr = (orc.cube_scatter(x, grid, cube) for x in (Qc, Kc, Vc))
    q, k, v = (usv.cube_gather(gu.up(x), grid, cube, seq_len=w.seq_len) for x in (Qr, Kr, Vr))
    S = usv.block_scores(q, k, seq_valid=w.seq_valid)
    idx, cnt = usv.select_topk(S, k=w.keep, seq_valid=w.seq_valid)
    o = usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, out_dtype=torch.float32)
    o_raster = gu.down(usv.cube_scatter(o, grid, cube))
    # oracle on the same path, taking the GPU's own fp32 scores for the selection
    Qo, Ko, Vo = (orc.cube_gather(synth.as_f32(x), grid, cube, w.seq_len) for x in (Qr, Kr, Vr))
    gu.assert_f32_close(gu.down(S), orc.block_scores(Qo, Ko, w.seq_valid))
    ridx, rcnt = orc.select_topk(gu.down(S), w.keep, w.seq_valid)
    np.testing.assert_array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_array_equal(cnt.cpu().numpy(), rcnt)
    ref = orc.cube_scatter(orc.block_sparse_attn(Qo, Ko, Vo, ridx, rcnt, w.seq_valid)[0], grid, cube)
    gu.assert_attn_close(o_raster, ref, "bf16", "raster pipeline")


@pytest.mark.parametrize("grid,Hh,dtype", [((21, 30, 52), 12, "bf16"), ((21, 30, 52), 12, "f32"), ((21, 45, 80), 40, "bf16")],
                         ids=["480p_bf16", "480p_f32_output", "720p_bf16"])
def test_full_size_grids_bit_exact(usv, grid, Hh, dtype):
    """The benchmark grids with all heads, in the launch configuration bench.py times (contiguous
    [1, Hh, Nv, 128]); the oracle redoes a sample of heads in full, the rest is covered by the round trip."""
    cube, d = (4, 4, 4), 128
    Nv = grid[0] * grid[1] * grid[2]
    N = -(-Nv // 64) * 64
    rng = np.random.default_rng([3, *grid])
    X = bits(rng, (1, Hh, Nv, d), dtype)
    x = to_dev(X)
    y = usv.cube_gather(x, grid, cube, seq_len=N)
    back = usv.cube_scatter(y, grid, cube)
    assert torch.equal(back.view(torch.int16 if dtype == "bf16" else torch.int32),
                       x.view(torch.int16 if dtype == "bf16" else torch.int32))
    order = orc.cube_token_order(grid, cube)
    for h in sorted(set(rng.choice(Hh, size=3, replace=False).tolist()) | {0, Hh - 1}):
        got = to_bits(y[0, h])
        np.testing.assert_array_equal(got[:Nv], X[0, h][order])
        assert not got[Nv:].any()
