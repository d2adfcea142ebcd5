"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares,
and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2512_05754_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000  # aligned, non-null; never dereferenced because validation fails first


def declared_functions():
    text = open(os.path.join(ROOT, "include", "usv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(usv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTED_SYMBOLS)
    for n in names:
        assert getattr(L, n) is not None


def test_header_is_plain_c(tmp_path):
    """include/usv.h is a C header: it must compile as C99 with no C++ and no torch types."""
    import shutil
    import subprocess

    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "hdr.c"
    src.write_text('#include "usv.h"\nint main(void) { usv_shape s; usv_raster r; (void)s; (void)r; return (int)USV_OK; }\n')
    res = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                          "-fsyntax-only", str(src)], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr


def shape(**kw):
    base = dict(batch=1, heads=2, seq_len=1024, seq_valid=1024, head_dim=64, block=64, dtype=binding.USV_F32)
    base.update(kw)
    return binding.UsvShape(**base)


def test_workspace_bytes():
    L = binding.lib()
    assert L.usv_workspace_bytes(ctypes.byref(shape())) == 2 * 2 * 16 * 64 * 4
    assert L.usv_workspace_bytes(ctypes.byref(shape(block=32))) == 0
    assert L.usv_workspace_bytes(None) == 0
    assert binding.workspace_bytes(1, 12, 32768, 32760, 128, "bf16") == 2 * 12 * 512 * 128 * 4


@pytest.mark.parametrize(
    "kw,status",
    [
        (dict(block=32), "USV_ERR_UNSUPPORTED"),
        (dict(head_dim=96), "USV_ERR_UNSUPPORTED"),
        (dict(dtype=7), "USV_ERR_UNSUPPORTED"),
        (dict(seq_len=1000), "USV_ERR_INVALID_ARG"),
        (dict(seq_valid=0), "USV_ERR_INVALID_ARG"),
        (dict(seq_valid=1025), "USV_ERR_INVALID_ARG"),
        (dict(batch=0), "USV_ERR_INVALID_ARG"),
        (dict(seq_len=64 * 4097, seq_valid=64), "USV_ERR_UNSUPPORTED"),
    ],
)
def test_bad_shapes_are_rejected_before_launch(kw, status):
    L = binding.lib()
    sh = shape(**kw)
    st = L.usv_block_scores(FAKE, FAKE, ctypes.byref(sh), FAKE, FAKE, 1 << 30, None)
    assert L.usv_status_string(st).decode() == status
    assert L.usv_last_error().decode() != ""
    st = L.usv_block_sparse_attn(FAKE, FAKE, FAKE, ctypes.byref(sh), FAKE, FAKE, 4, 0.0, sh.dtype, FAKE, None, None)
    assert L.usv_status_string(st).decode() == status


def test_bad_pointers_workspace_and_budgets():
    L = binding.lib()
    sh = ctypes.byref(shape())
    name = lambda st: L.usv_status_string(st).decode()
    assert name(L.usv_block_scores(None, FAKE, sh, FAKE, FAKE, 1 << 20, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_block_scores(FAKE + 4, FAKE, sh, FAKE, FAKE, 1 << 20, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_block_scores(FAKE, FAKE, sh, FAKE, FAKE, 100, None)) == "USV_ERR_WORKSPACE"
    assert name(L.usv_block_scores(FAKE, FAKE, sh, FAKE, None, 1 << 20, None)) == "USV_ERR_WORKSPACE"
    assert "bytes" in L.usv_last_error().decode()
    # top-k: k and kmax ranges
    assert name(L.usv_select_topk(FAKE, sh, 0, None, 4, FAKE, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_select_topk(FAKE, sh, 5, None, 4, FAKE, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_select_topk(FAKE, sh, 4, None, 17, FAKE, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_select_topk(FAKE, sh, 4, None, 0, FAKE, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_select_topk(None, sh, 4, None, 4, FAKE, FAKE, None)) == "USV_ERR_INVALID_ARG"
    # attention: kmax, scale, out_dtype
    a = lambda kmax, scale, od: name(
        L.usv_block_sparse_attn(FAKE, FAKE, FAKE, sh, FAKE, FAKE, kmax, scale, od, FAKE, None, None)
    )
    assert a(0, 0.0, 0) == "USV_ERR_INVALID_ARG"
    assert a(17, 0.0, 0) == "USV_ERR_INVALID_ARG"
    assert a(4, float("nan"), 0) == "USV_ERR_INVALID_ARG"
    assert a(4, 0.0, binding.USV_BF16) == "USV_ERR_UNSUPPORTED"  # fp32 inputs cannot produce bf16 output
    assert L.usv_status_string(99).decode() == "USV_ERR_UNKNOWN"


def test_binding_refuses_cpu_tensors():
    import torch

    x = torch.zeros(1, 1, 64, 64)
    with pytest.raises(TypeError, match="GPU tensor"):
        binding.block_scores(x, x)


# --------------------------------------------------------------------------- #
# raster <-> cube-major order: the closed form the kernel uses, checked on the host
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("grid,cube", [
    ((21, 30, 52), (4, 4, 4)), ((21, 45, 80), (4, 4, 4)), ((8, 8, 8), (4, 4, 4)), ((5, 6, 7), (4, 4, 4)),
    ((1, 9, 9), (4, 4, 4)), ((3, 3, 3), (4, 4, 4)), ((7, 4, 4), (4, 4, 4)), ((4, 4, 3), (4, 4, 4)),
    ((3, 17, 19), (1, 8, 8)), ((5, 9, 20), (2, 4, 8)), ((2, 2, 130), (1, 1, 64)), ((9, 5, 6), (16, 2, 2)),
])
def test_cube_token_order_closed_form_equals_oracle_enumeration(grid, cube):
    """usv_cube_token_order evaluates the same closed-form position function as the kernel; the
    oracle walks the cubes one by one."""
    import numpy as np

    from oracle import usv_oracle as orc

    got = binding.cube_token_order(grid, cube)
    np.testing.assert_array_equal(got.astype(np.int64), orc.cube_token_order(grid, cube))


@pytest.mark.parametrize(
    "grid,shape_kw,strides,status",
    [
        ((4, 4, 4, 4, 4, 2), {}, None, "USV_ERR_UNSUPPORTED"),            # cube of 32 tokens
        ((4, 4, 4, 0, 4, 4), {}, None, "USV_ERR_INVALID_ARG"),            # zero cube extent
        ((0, 4, 4, 4, 4, 4), {}, None, "USV_ERR_INVALID_ARG"),            # empty grid
        ((4, 4, 5, 4, 4, 4), {}, None, "USV_ERR_INVALID_ARG"),            # 80 tokens but seq_valid = 64
        ((4, 4, 4, 4, 4, 4), {}, (64 * 64, 64, 32), "USV_ERR_INVALID_ARG"),   # token stride < head_dim
        ((4, 4, 4, 4, 4, 4), {}, (64 * 64, 64 * 64, 66), "USV_ERR_INVALID_ARG"),  # rows not 16-byte aligned
        ((4, 4, 4, 4, 4, 4), dict(head_dim=96), None, "USV_ERR_UNSUPPORTED"),
    ],
)
def test_cube_move_rejects_bad_arguments_before_launch(grid, shape_kw, strides, status):
    L = binding.lib()
    sh = shape(seq_len=64, seq_valid=64, **shape_kw)
    g = binding.UsvGrid(*grid)
    st = None if strides is None else ctypes.byref(binding.UsvStrides(*strides))
    for rc in (L.usv_cube_gather(FAKE, st, ctypes.byref(sh), ctypes.byref(g), FAKE, None),
               L.usv_cube_scatter(FAKE, ctypes.byref(sh), ctypes.byref(g), FAKE, st, None)):
        assert L.usv_status_string(rc).decode() == status
    assert L.usv_last_error()


def test_cube_move_rejects_null_and_misaligned_pointers():
    L = binding.lib()
    sh, g = shape(seq_len=64, seq_valid=64), binding.UsvGrid(4, 4, 4, 4, 4, 4)
    assert L.usv_cube_gather(None, None, ctypes.byref(sh), ctypes.byref(g), FAKE, None) == 1
    assert L.usv_cube_gather(FAKE, None, ctypes.byref(sh), ctypes.byref(g), FAKE + 4, None) == 1
    assert L.usv_cube_scatter(FAKE, ctypes.byref(sh), None, FAKE, None, None) == 1
    assert L.usv_cube_token_order(ctypes.byref(g), None) == 1


def test_raster_entry_points_reject_bad_arguments_before_launch():
    L = binding.lib()
    name = lambda rc: L.usv_status_string(rc).decode()
    sh = shape(seq_len=64, seq_valid=64, head_dim=128, dtype=binding.USV_BF16)
    g = binding.UsvGrid(4, 4, 4, 4, 4, 4)
    zero = binding.UsvStrides(0, 0, 0)
    view = binding.UsvRaster(FAKE, zero, zero)
    need = L.usv_workspace_bytes(ctypes.byref(sh))
    bf16, f32 = binding.USV_BF16, binding.USV_F32
    # usv_cube_order
    assert name(L.usv_cube_order(ctypes.byref(sh), ctypes.byref(g), None, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_cube_order(ctypes.byref(sh), ctypes.byref(binding.UsvGrid(4, 4, 5, 4, 4, 4)), FAKE, None)) == "USV_ERR_INVALID_ARG"
    # usv_block_scores_raster
    assert name(L.usv_block_scores_raster(FAKE, FAKE, ctypes.byref(sh), None, FAKE, FAKE, need, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_block_scores_raster(FAKE, FAKE, ctypes.byref(sh), ctypes.byref(binding.UsvRaster(None, zero, zero)),
                                          FAKE, FAKE, need, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_block_scores_raster(FAKE, FAKE, ctypes.byref(sh), ctypes.byref(view), FAKE, FAKE, need - 1, None)) == "USV_ERR_WORKSPACE"
    short_rows = binding.UsvRaster(FAKE, binding.UsvStrides(2 * 64 * 128, 64 * 128, 64), zero)  # token stride < head_dim
    assert name(L.usv_block_scores_raster(FAKE, FAKE, ctypes.byref(sh), ctypes.byref(short_rows), FAKE, FAKE, need, None)) == "USV_ERR_INVALID_ARG"
    # usv_block_sparse_attn_raster
    args = lambda shp, vw, kmax=1, od=bf16, scale=0.0, out=FAKE: L.usv_block_sparse_attn_raster(
        FAKE, FAKE, FAKE, ctypes.byref(shp), ctypes.byref(vw), FAKE, FAKE, kmax, ctypes.c_float(scale), od, out, None, None)
    assert name(args(shape(seq_len=64, seq_valid=64, head_dim=128), view)) == "USV_ERR_UNSUPPORTED"      # fp32 inputs
    assert name(args(sh, view, od=7)) == "USV_ERR_UNSUPPORTED"
    assert name(args(sh, view, kmax=0)) == "USV_ERR_INVALID_ARG"
    assert name(args(sh, view, kmax=2)) == "USV_ERR_INVALID_ARG"                                          # kmax > blocks
    assert name(args(sh, view, scale=float("inf"))) == "USV_ERR_INVALID_ARG"
    assert name(args(sh, view, out=None)) == "USV_ERR_INVALID_ARG"
    big = shape(seq_len=1 << 18, seq_valid=1 << 18, head_dim=128, dtype=bf16)                             # 2^18 tokens x 16 KiB rows
    wide = binding.UsvRaster(FAKE, binding.UsvStrides(1 << 40, 128, 8192), zero)
    assert name(args(big, wide)) == "USV_ERR_UNSUPPORTED"
    assert b"2 GiB" in L.usv_last_error()
    # the second branch on raster tensors
    cneed = L.usv_coarse_workspace_bytes(ctypes.byref(sh))
    assert name(L.usv_coarse_attn_raster(FAKE, FAKE, ctypes.byref(sh), None, FAKE, FAKE, cneed, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_coarse_attn_raster(FAKE, FAKE, ctypes.byref(sh), ctypes.byref(view), FAKE, FAKE, cneed - 1, None)) == "USV_ERR_WORKSPACE"
    assert name(L.usv_coarse_attn_raster(None, FAKE, ctypes.byref(sh), ctypes.byref(view), FAKE, FAKE, cneed, None)) == "USV_ERR_INVALID_ARG"
    fused = lambda coarse, gf, gc: L.usv_block_sparse_attn_raster_fused(
        FAKE, FAKE, FAKE, ctypes.byref(sh), ctypes.byref(view), FAKE, FAKE, 1, ctypes.c_float(0.0), coarse, gf, gc, bf16, FAKE,
        None, None)
    assert name(fused(None, FAKE, None)) == "USV_ERR_INVALID_ARG"       # gates without the cube-level rows
    assert name(fused(FAKE + 4, None, None)) == "USV_ERR_INVALID_ARG"   # misaligned
    assert name(fused(FAKE, FAKE + 2, None)) == "USV_ERR_INVALID_ARG"


# --------------------------------------------------------------------------- #
# cube-level branch, fusion, selection flags
# --------------------------------------------------------------------------- #
def test_coarse_and_fuse_reject_bad_arguments_before_launch():
    L = binding.lib()
    sh = shape()
    need = L.usv_coarse_workspace_bytes(ctypes.byref(sh))
    assert need == 2 * 16 * 64 * 4
    assert L.usv_coarse_workspace_bytes(ctypes.byref(shape(head_dim=80))) == 0
    name = lambda rc: L.usv_status_string(rc).decode()
    assert name(L.usv_coarse_attn(FAKE, FAKE, ctypes.byref(sh), FAKE, FAKE, need - 1, None)) == "USV_ERR_WORKSPACE"
    assert name(L.usv_coarse_attn(FAKE, FAKE, ctypes.byref(sh), FAKE, None, need, None)) == "USV_ERR_WORKSPACE"
    assert name(L.usv_coarse_attn(None, FAKE, ctypes.byref(sh), FAKE, FAKE, need, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_coarse_attn(FAKE, FAKE, ctypes.byref(shape(block=32)), FAKE, FAKE, need, None)) == "USV_ERR_UNSUPPORTED"
    f32, bf16 = binding.USV_F32, binding.USV_BF16
    assert name(L.usv_fuse_outputs(FAKE, 5, FAKE, None, None, ctypes.byref(sh), f32, FAKE + 64, None)) == "USV_ERR_UNSUPPORTED"
    assert name(L.usv_fuse_outputs(FAKE, f32, FAKE, None, None, ctypes.byref(sh), bf16, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_fuse_outputs(FAKE, f32, FAKE, FAKE + 2, None, ctypes.byref(sh), f32, FAKE + 64, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_fuse_outputs(FAKE, f32, None, None, None, ctypes.byref(sh), f32, FAKE + 64, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_select_topk_ex(FAKE, ctypes.byref(sh), 2, None, 4, 6, FAKE, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert b"flag" in L.usv_last_error()


# --------------------------------------------------------------------------- #
# entropy-aware allocation: the host helper against the oracle
# --------------------------------------------------------------------------- #
def test_entropy_allocate_matches_oracle():
    import numpy as np

    from oracle import usv_oracle as orc

    rng = np.random.default_rng(0)
    for L, gamma, bar, lo, hi in [(30, 2.0, 0.9, 0.5, 0.98), (1, 1.0, 0.8, 0.0, 1.0), (7, 4.0, 0.95, 0.9, 0.99),
                                  (12, 1.5, 0.5, 0.0, 10.0)]:
        h = rng.uniform(0, 1, size=L).astype(np.float32)
        got = binding.entropy_allocate(h, bar, gamma, lo, hi)
        ref = orc.entropy_allocate(h.astype(np.float64), bar, gamma, lo, hi)
        np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-7)
    # without clipping the layer mean is the base sparsity
    h = rng.uniform(0, 1, size=16).astype(np.float32)
    assert abs(binding.entropy_allocate(h, 0.8, 2.0, 0.0, 100.0).mean() - 0.8) < 1e-6
    # all layers at entropy 1: no weight anywhere, the base schedule is kept
    for hs, bar, lo, hi in [([1.0, 1.0], 0.7, 0.0, 1.0), ([1.0] * 5, 0.7, 0.0, 0.6), ([1.0], 0.2, 0.3, 0.9)]:
        got = binding.entropy_allocate(hs, bar, 2.0, lo, hi)
        ref = orc.entropy_allocate(np.asarray(hs, dtype=np.float64), bar, 2.0, lo, hi)
        assert np.isfinite(ref).all()
        np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-7)


def test_entropy_calls_reject_bad_arguments():
    L = binding.lib()
    name = lambda rc: L.usv_status_string(rc).decode()
    sh = shape()
    need = L.usv_entropy_workspace_bytes(ctypes.byref(sh))
    assert need == 2 * 1 * 16 * 4  # B*Hh = 2, one 32-row tile of 16 cubes
    assert name(L.usv_attn_entropy(FAKE, ctypes.byref(sh), FAKE, FAKE, need - 1, None)) == "USV_ERR_WORKSPACE"
    assert name(L.usv_attn_entropy(FAKE, ctypes.byref(sh), None, FAKE, need, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_attn_entropy(None, ctypes.byref(sh), FAKE, FAKE, need, None)) == "USV_ERR_INVALID_ARG"
    buf = (ctypes.c_float * 3)(0.1, 0.2, 1.5)
    out = (ctypes.c_float * 3)()
    assert name(L.usv_entropy_allocate(buf, 3, 0.8, 2.0, 0.0, 1.0, out)) == "USV_ERR_INVALID_ARG"  # entropy > 1
    buf[2] = 0.5
    assert name(L.usv_entropy_allocate(buf, 3, 0.8, 0.5, 0.0, 1.0, out)) == "USV_ERR_INVALID_ARG"  # gamma < 1
    assert name(L.usv_entropy_allocate(buf, 3, 0.8, 2.0, 0.9, 0.1, out)) == "USV_ERR_INVALID_ARG"  # min > max
    assert name(L.usv_entropy_allocate(buf, 0, 0.8, 2.0, 0.0, 1.0, out)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_entropy_allocate(None, 3, 0.8, 2.0, 0.0, 1.0, out)) == "USV_ERR_INVALID_ARG"
    assert L.usv_entropy_allocate(buf, 3, 0.8, 2.0, 0.0, 1.0, out) == 0


# --------------------------------------------------------------------------- #
# token merging: argument validation
# --------------------------------------------------------------------------- #
def test_merge_calls_reject_bad_arguments_before_launch():
    L = binding.lib()
    name = lambda rc: L.usv_status_string(rc).decode()
    g = binding.UsvGrid(4, 6, 8, 2, 2, 2)  # 192 tokens, 24 destinations, 168 sources
    ok = shape(seq_len=128, seq_valid=100)   # r = 92
    assert L.usv_merge_workspace_bytes(ctypes.byref(ok), ctypes.byref(g)) == 1 * 192 * 65 * 4
    few = shape(seq_len=64, seq_valid=23)    # fewer rows than destinations
    many = shape(seq_len=256, seq_valid=193)  # more rows than tokens
    for bad in (few, many):
        assert L.usv_merge_workspace_bytes(ctypes.byref(bad), ctypes.byref(g)) == 0
        assert name(L.usv_merge_plan(FAKE, FAKE, ctypes.byref(bad), ctypes.byref(g), FAKE, FAKE, None, 0, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_merge_plan(FAKE, FAKE, ctypes.byref(ok), None, FAKE, FAKE, None, 0, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_merge_plan(None, FAKE, ctypes.byref(ok), ctypes.byref(g), FAKE, FAKE, None, 0, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_merge_plan(FAKE, None, ctypes.byref(ok), ctypes.byref(g), FAKE, FAKE, None, 0, None)) == "USV_ERR_INVALID_ARG"
    # the chip-wide selection's scratch: state, two 4096-bin count arrays, and 256 + 2 ints per slice of 2048 tokens
    need_plan = L.usv_merge_plan_workspace_bytes(ctypes.byref(ok), ctypes.byref(g))
    assert need_plan == (8 + 2 * 4096 + 1 * 258) * 4
    assert L.usv_merge_plan_workspace_bytes(ctypes.byref(few), ctypes.byref(g)) == 0
    assert name(L.usv_merge_plan(FAKE, FAKE, ctypes.byref(ok), ctypes.byref(g), FAKE, FAKE, FAKE, need_plan - 1, None)) == "USV_ERR_WORKSPACE"
    zero = binding.UsvGrid(4, 6, 8, 2, 0, 2)
    assert name(L.usv_merge_apply(FAKE, ctypes.byref(ok), ctypes.byref(zero), FAKE, FAKE, FAKE, None)) == "USV_ERR_INVALID_ARG"
    need = L.usv_merge_workspace_bytes(ctypes.byref(ok), ctypes.byref(g))
    assert name(L.usv_merge_similarity(FAKE, ctypes.byref(ok), ctypes.byref(g), FAKE, FAKE, FAKE, need - 1, None)) == "USV_ERR_WORKSPACE"
    assert name(L.usv_unmerge_apply(FAKE, ctypes.byref(ok), ctypes.byref(g), FAKE + 2, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_merge_apply(FAKE, ctypes.byref(shape(seq_len=128, seq_valid=100, head_dim=48)), ctypes.byref(g),
                                  FAKE, FAKE, FAKE, None)) == "USV_ERR_UNSUPPORTED"


def test_fused_attention_rejects_gates_without_coarse():
    L = binding.lib()
    sh = shape(dtype=binding.USV_BF16)
    args = (FAKE, FAKE, FAKE, ctypes.byref(sh), FAKE, FAKE, 4, ctypes.c_float(0.0))
    rc = L.usv_block_sparse_attn_fused(*args, None, FAKE, None, binding.USV_BF16, FAKE, None, None)
    assert L.usv_status_string(rc).decode() == "USV_ERR_INVALID_ARG" and b"coarse" in L.usv_last_error()
    rc = L.usv_block_sparse_attn_fused(*args, FAKE + 8, None, None, binding.USV_BF16, FAKE, None, None)
    assert L.usv_status_string(rc).decode() == "USV_ERR_INVALID_ARG"


def _run_bench(*args):
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    return subprocess.run([sys.executable, os.path.join(root, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300)


def test_bench_refuses_more_than_one_gpu():
    r = _run_bench("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_bench_fails_loudly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("checks the no-GPU error path")
    r = _run_bench("--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "no CPU fallback" in (r.stdout + r.stderr)
    assert "{" not in r.stdout  # no result line is printed


def test_traffic_figures_belong_to_the_kernel_sources_in_the_tree():
    """profiles/traffic.json entries carry a digest of the kernel sources they were measured with: an entry that is
    older than its kernel must be re-measured (or bench.py reports it as null)."""
    from paper_2512_05754_amd import traffic

    assert traffic.check() == 0, "stale entry in profiles/traffic.json: run the rocprofv3 passes again and record them"


# --------------------------------------------------------------------------- #
# the C ABI from C: tools/usv_demo.c compiles as C99 against include/usv.h and links against libusv.so
# --------------------------------------------------------------------------- #
def test_c_demo_builds_and_reports_usage():
    import subprocess

    from paper_2512_05754_amd.build import build_demo

    binding.lib()  # the program links against libusv.so: make sure it exists
    exe = build_demo(verbose=False)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert res.returncode == 1 and "usage" in res.stderr


# --------------------------------------------------------------------------- #
# work order, ordered attention, static stage 1, padded cube order: validation before any launch
# --------------------------------------------------------------------------- #
def test_order_static_and_padded_cube_calls_reject_bad_arguments():
    L = binding.lib()
    name = lambda rc: L.usv_status_string(rc).decode()
    ok = shape()
    nb = ok.seq_len // 64
    # usv_attn_work_order: idx may be NULL (lengths only); cnt, the table and kmax are checked
    assert name(L.usv_attn_work_order(None, None, ctypes.byref(ok), 4, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_attn_work_order(None, FAKE, ctypes.byref(ok), 4, None, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_attn_work_order(FAKE + 4, FAKE, ctypes.byref(ok), 4, FAKE, None)) == "USV_ERR_INVALID_ARG"
    for kmax in (0, nb + 1):
        assert name(L.usv_attn_work_order(None, FAKE, ctypes.byref(ok), kmax, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_attn_work_order(None, FAKE, None, 4, FAKE, None)) == "USV_ERR_INVALID_ARG"
    # usv_block_sparse_attn_ordered: a misaligned table is refused; everything else as usv_block_sparse_attn
    args = (FAKE, FAKE, FAKE, ctypes.byref(ok), FAKE, FAKE, 4)
    assert name(L.usv_block_sparse_attn_ordered(*args, FAKE + 4, 0.0, ok.dtype, FAKE, None, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_block_sparse_attn_ordered(*args, FAKE, float("nan"), ok.dtype, FAKE, None, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_block_sparse_attn_ordered(*args, FAKE, 0.0, ok.dtype, None, None, None)) == "USV_ERR_INVALID_ARG"
    # usv_block_scores_static: pointers and shape are checked like usv_block_scores; the size limit has its own status
    assert name(L.usv_block_scores_static(None, FAKE, ctypes.byref(ok), FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_block_scores_static(FAKE, FAKE, ctypes.byref(ok), None, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_block_scores_static(FAKE, FAKE, ctypes.byref(shape(block=32)), FAKE, None)) == "USV_ERR_UNSUPPORTED"
    big = shape(batch=2, heads=33, seq_len=1024 * 64, seq_valid=1024 * 64, head_dim=128)
    assert L.usv_workspace_bytes(ctypes.byref(big)) > (64 << 20)
    assert name(L.usv_block_scores_static(FAKE, FAKE, ctypes.byref(big), FAKE, None)) == "USV_ERR_WORKSPACE"
    # usv_cube_count / usv_cube_order_padded
    g = binding.UsvGrid(21, 30, 52, 4, 4, 4)
    assert L.usv_cube_count(ctypes.byref(g)) == 6 * 8 * 13
    assert L.usv_cube_count(ctypes.byref(binding.UsvGrid(21, 30, 52, 4, 0, 4))) == 0
    assert L.usv_cube_count(None) == 0
    assert name(L.usv_cube_order_padded(None, FAKE, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_cube_order_padded(ctypes.byref(g), None, FAKE, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_cube_order_padded(ctypes.byref(g), FAKE, FAKE + 2, None)) == "USV_ERR_INVALID_ARG"
    assert name(L.usv_cube_order_padded(ctypes.byref(binding.UsvGrid(4, 4, 4, 8, 8, 8)), FAKE, FAKE, None)) == "USV_ERR_UNSUPPORTED"
