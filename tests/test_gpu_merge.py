"""GPU parity of token merging (Section 3.3) against the oracle.

The similarities are compared at the fp32 bound; the plan (which sources merge, where every token
reads back) is compared bit-exactly, the oracle selecting from the SAME fp32 similarities the GPU
produced; merged features at the fp32 bound (bf16 storage: one rounding); the unmerge is byte work."""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import usv_oracle as orc
from paper_2512_05754_amd import synth

pytestmark = pytest.mark.gpu

CASES = [
    # grid, merge block, B, Hh, d, dtype
    ((4, 6, 8), (2, 2, 2), 2, 3, 64, "f32"),
    ((5, 7, 9), (2, 2, 4), 1, 4, 128, "bf16"),     # cut blocks on every axis
    ((3, 10, 13), (1, 2, 2), 2, 2, 128, "f32"),
    ((2, 33, 70), (2, 4, 4), 1, 5, 64, "bf16"),    # 4620 tokens: several sweeps of the 1024-thread selection
    ((6, 4, 4), (4, 4, 4), 1, 2, 128, "bf16"),     # the attention cube as the merge block
]


def make(rng, shape, dtype, smooth=None):
    x = rng.standard_normal(shape).astype(np.float32)
    if smooth is not None:
        x = x + 2.0 * smooth
    return synth.f32_to_bf16_bits(x) if dtype == "bf16" else x


def expected_blk(grid, mb):
    """The partition array from the oracle's partition: rank of each token's destination among the destinations
    (ascending raster index), bit 31 at the destinations."""
    dst = orc.merge_partition(grid, mb)
    n = len(dst)
    dsts = np.nonzero(dst == np.arange(n))[0]
    rank = np.searchsorted(dsts, dst).astype(np.int64)
    rank[dst == np.arange(n)] |= 0x80000000
    return rank.astype(np.uint32).view(np.int32)


def both_plans(usv, u, blk, grid, mb, r):
    """usv_merge_plan both ways: one workgroup per batch element (no workspace) and the radix select spread over the chip
    (workspace, handed over full of garbage: nothing in it is assumed clear).  The two must agree bit for bit."""
    one = usv.merge_plan(u, blk, grid, mb, r, workspace=False)
    ws = torch.full((usv.merge_plan_workspace_bytes(u.shape[0], grid, mb, r),), 0xA5, dtype=torch.uint8, device=u.device)
    wide = usv.merge_plan(u, blk, grid, mb, r, workspace=ws)
    assert torch.equal(one[0], wide[0]) and torch.equal(one[1], wide[1]), f"r={r}: the two selections differ"
    return wide


def bf16_round_ok(got, ref):
    return np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * np.maximum(1, np.abs(ref))


@pytest.mark.parametrize("grid,mb,B,Hh,d,dtype", CASES, ids=lambda v: str(v).replace(" ", ""))
def test_merge_pipeline(usv, grid, mb, B, Hh, d, dtype):
    rng = np.random.default_rng([61, *grid, d])
    N = grid[0] * grid[1] * grid[2]
    base = rng.standard_normal((B, 1, N, d)).astype(np.float32)  # shared by the heads: descriptors do not average out
    K = make(rng, (B, Hh, N, d), dtype, base)
    X = make(rng, (B, Hh, N, d), dtype)
    Kf, Xf = synth.as_f32(K), synth.as_f32(X)
    u, blk = usv.merge_similarity(gu.up(K), grid, mb)
    u_h = gu.down(u)
    u_ref = orc.merge_similarity(Kf, grid, mb)
    np.testing.assert_array_equal(blk.cpu().numpy(), expected_blk(grid, mb))
    assert np.array_equal(np.isneginf(u_h), np.isneginf(u_ref))
    gu.assert_f32_close(u_h, u_ref, "similarity")
    n_src = int((~np.isneginf(u_ref[0])).sum())
    for r in sorted({0, 1, n_src // 3, n_src // 2, n_src}):
        row_of, src_of = both_plans(usv, u, blk, grid, mb, r)
        rr, rs = orc.merge_plan(u_h, grid, mb, r)
        np.testing.assert_array_equal(row_of.cpu().numpy(), rr)
        np.testing.assert_array_equal(src_of.cpu().numpy(), rs)
        Np = -(-(N - r) // 64) * 64 + 64
        y = usv.merge_apply(gu.up(X), grid, mb, row_of, src_of, seq_len=Np)
        y_ref = orc.merge_apply(Xf, rr, rs, Np)
        y_h = gu.down(y)
        assert not y_h[:, :, N - r:].any()
        if dtype == "f32":
            gu.assert_f32_close(y_h, y_ref, f"merge r={r}")
        else:
            ok = bf16_round_ok(y_h, y_ref)
            assert ok.all(), f"merge r={r}: {(~ok).sum()} elements beyond one bf16 rounding"
        z = usv.unmerge_apply(y, grid, mb, row_of, N - r)
        z_ref = orc.unmerge_apply(y_h, rr)
        np.testing.assert_array_equal(gu.down(z), z_ref)


def test_merge_plan_ties_and_special_values(usv):
    """Engineered similarities: many exact ties across the sweep boundary of the selection, signed zeros,
    NaN (ranks lowest), several batch elements with different values."""
    grid, mb = (3, 20, 40), (1, 2, 2)
    N = 2400
    rng = np.random.default_rng(7)
    dst = orc.merge_partition(grid, mb)
    u = np.round(rng.standard_normal((3, N)) * 2).astype(np.float32) / 4  # heavy ties
    u[1, ::7] = -0.0
    u[1, 3::11] = 0.0
    u[2, 5::13] = np.nan
    u[:, dst == np.arange(N)] = -np.inf
    n_src = int((dst != np.arange(N)).sum())
    for r in (1, 37, 1000, 1024, 1500, n_src - 1, n_src):
        row_of, src_of = both_plans(usv, gu.up(u), gu.up(expected_blk(grid, mb)), grid, mb, r)
        rr, rs = orc.merge_plan(u, grid, mb, r)
        np.testing.assert_array_equal(row_of.cpu().numpy(), rr)
        np.testing.assert_array_equal(src_of.cpu().numpy(), rs)


def test_merge_then_attention_then_unmerge(usv):
    """Raster Q/K/V -> merge (half of the tokens) -> three-stage hot path on the merged sequence -> unmerge,
    against the oracle doing the same with the GPU's own similarities and scores."""
    grid, mb = (4, 8, 12), (2, 2, 2)
    B, Hh, d, N = 1, 2, 128, 384
    rng = np.random.default_rng(71)
    base = rng.standard_normal((B, 1, N, d)).astype(np.float32)
    Q, K, V = (make(rng, (B, Hh, N, d), "bf16", base) for _ in range(3))
    r = N // 2 - 5  # 197 merged rows: a ragged tail inside the last 64-row block
    u, blk = usv.merge_similarity(gu.up(K), grid, mb)
    row_of, src_of = usv.merge_plan(u, blk, grid, mb, r)
    q, k, v = (usv.merge_apply(gu.up(x), grid, mb, row_of, src_of) for x in (Q, K, V))
    Nm = N - r
    S = usv.block_scores(q, k, seq_valid=Nm)
    idx, cnt = usv.select_topk(S, k=2, seq_valid=Nm)
    o = usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=Nm, out_dtype=torch.float32)
    out = gu.down(usv.unmerge_apply(o, grid, mb, row_of, Nm))
    # oracle: same plan from the same u; merged tensors as the GPU stored them (bf16), then fp64 throughout
    rr, rs = orc.merge_plan(gu.down(u), grid, mb, r)
    np.testing.assert_array_equal(row_of.cpu().numpy(), rr)
    qm, km, vm = gu.down(q).astype(np.float64), gu.down(k).astype(np.float64), gu.down(v).astype(np.float64)
    for got, raw in ((qm, Q), (km, K), (vm, V)):
        assert bf16_round_ok(got, orc.merge_apply(synth.as_f32(raw), rr, rs, q.shape[2])).all()
    ridx, rcnt = orc.select_topk(gu.down(S), 2, Nm)
    np.testing.assert_array_equal(idx.cpu().numpy(), ridx)
    ref = orc.unmerge_apply(orc.block_sparse_attn(qm, km, vm, ridx, rcnt, Nm)[0], rr)
    gu.assert_attn_close(out, ref, "bf16", "merged pipeline")


def test_full_size_480p_half_merged(usv):
    """The benchmark shape of bench.py --path merge: 21 x 30 x 52 tokens, 12 heads, 2x2x2 blocks, half of the
    tokens merged.  Plan bit-exact on all 32760 tokens; features on sampled heads; unmerge bit-exact."""
    grid, mb, Hh, d = (21, 30, 52), (2, 2, 2), 12, 128
    N = 32760
    r = N // 2
    gen = torch.Generator(device=gu.DEV).manual_seed(5)
    base = torch.randn((1, 1, N, d), device=gu.DEV, generator=gen)
    k = (torch.randn((1, Hh, N, d), device=gu.DEV, generator=gen) + 2 * base).to(torch.bfloat16)
    x = torch.randn((1, Hh, N, d), device=gu.DEV, generator=gen).to(torch.bfloat16)
    u, blk = usv.merge_similarity(k, grid, mb)
    u_h = gu.down(u)
    gu.assert_f32_close(u_h, orc.merge_similarity(gu.down(k).astype(np.float64), grid, mb), "similarity 480p")
    row_of, src_of = both_plans(usv, u, blk, grid, mb, r)
    rr, rs = orc.merge_plan(u_h, grid, mb, r)
    np.testing.assert_array_equal(row_of.cpu().numpy(), rr)
    np.testing.assert_array_equal(src_of.cpu().numpy(), rs)
    y = usv.merge_apply(x, grid, mb, row_of, src_of)
    assert y.shape[2] == 16384
    for h in (0, 7):
        ref = orc.merge_apply(gu.down(x[:, h:h + 1]).astype(np.float64), rr, rs, 16384)
        ok = bf16_round_ok(gu.down(y[:, h:h + 1]), ref)
        assert ok.all(), f"head {h}: {(~ok).sum()} elements beyond one bf16 rounding"
    z = usv.unmerge_apply(y, grid, mb, row_of, N - r)
    idx = torch.from_numpy(rr[0].astype(np.int64)).to(gu.DEV)
    assert torch.equal(z.view(torch.int16), y[:, :, idx, :].view(torch.int16))


@pytest.mark.parametrize("grid,mb", [((21, 45, 80), (2, 2, 2)), ((24, 60, 64), (1, 2, 2)), ((9, 100, 111), (4, 4, 4))],
                         ids=["720p_75600_tokens", "92160_tokens", "99900_tokens_cut_blocks"])
def test_merge_plan_large_token_counts(usv, grid, mb):
    """Token counts beyond 32768 (keys in 80 registers per thread) and beyond 81920 (keys re-read from memory
    in every pass): plan bit-exact on engineered similarities with ties, two batch elements."""
    N = grid[0] * grid[1] * grid[2]
    rng = np.random.default_rng([9, N])
    dst = orc.merge_partition(grid, mb)
    blk = expected_blk(grid, mb)
    u = (np.round(rng.standard_normal((2, N)) * 64) / 256).astype(np.float32)  # ~600 distinct values: ties everywhere
    u[1] = rng.standard_normal(N).astype(np.float32)                             # and a row without ties
    u[:, dst == np.arange(N)] = -np.inf
    n_src = int((dst != np.arange(N)).sum())
    u[0, 5::97] = np.nan
    u[0, 11::89] = -0.0
    u[0, 17::83] = np.inf
    u[:, dst == np.arange(N)] = -np.inf
    for r in (N // 2 if N // 2 <= n_src else n_src, 4097, 1, n_src - 1, n_src, 0):
        row_of, src_of = both_plans(usv, gu.up(u), gu.up(blk), grid, mb, r)
        rr, rs = orc.merge_plan(u, grid, mb, r)
        np.testing.assert_array_equal(row_of.cpu().numpy(), rr)
        np.testing.assert_array_equal(src_of.cpu().numpy(), rs)
