"""ctypes binding of libusv.so: argument marshalling only, every step runs in the HIP kernels.

Functions mirror the C ABI (include/usv.h) name for name.  Tensors are torch CUDA(ROCm)
tensors used purely as device memory; work is enqueued on torch's current stream.
There is no CPU fallback: a missing library or a CPU tensor raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
BLOCK = 64
USV_F32, USV_BF16 = 0, 1

EXPORTED_SYMBOLS = (
    "usv_workspace_bytes",
    "usv_block_scores",
    "usv_block_scores_static",
    "usv_select_topk",
    "usv_select_topk_ex",
    "usv_coarse_workspace_bytes",
    "usv_coarse_attn",
    "usv_fuse_outputs",
    "usv_entropy_workspace_bytes",
    "usv_attn_entropy",
    "usv_entropy_allocate",
    "usv_block_sparse_attn",
    "usv_block_sparse_attn_fused",
    "usv_attn_work_order",
    "usv_block_sparse_attn_ordered",
    "usv_merge_workspace_bytes",
    "usv_merge_similarity",
    "usv_merge_plan",
    "usv_merge_plan_workspace_bytes",
    "usv_merge_apply",
    "usv_unmerge_apply",
    "usv_cube_order",
    "usv_cube_count",
    "usv_cube_order_padded",
    "usv_block_scores_raster",
    "usv_block_sparse_attn_raster",
    "usv_coarse_attn_raster",
    "usv_block_sparse_attn_raster_fused",
    "usv_cube_token_order",
    "usv_cube_gather",
    "usv_cube_scatter",
    "usv_status_string",
    "usv_last_error",
)


class UsvError(RuntimeError):
    def __init__(self, status: int, name: str, message: str):
        super().__init__(f"{name} ({status}): {message}")
        self.status = status
        self.status_name = name


class UsvShape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32),
        ("heads", ctypes.c_int32),
        ("seq_len", ctypes.c_int32),
        ("seq_valid", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("block", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
    ]


class UsvGrid(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "H", "W", "ct", "ch", "cw")]


class UsvStrides(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("batch", "head", "token")]


class UsvRaster(ctypes.Structure):
    _fields_ = [("order", ctypes.c_void_p), ("in_strides", UsvStrides), ("out_strides", UsvStrides),
                ("block_valid", ctypes.c_void_p), ("work_order", ctypes.c_void_p)]


def lib_path() -> str:
    return os.path.join(PKG_DIR, "libusv.so")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libusv.so (building it first only if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        from .build import build_library

        build_library(verbose=False)
    L = ctypes.CDLL(path)
    vp, i32, sz, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t, ctypes.c_float
    sp = ctypes.POINTER(UsvShape)
    L.usv_workspace_bytes.restype, L.usv_workspace_bytes.argtypes = sz, [sp]
    L.usv_block_scores.restype, L.usv_block_scores.argtypes = i32, [vp, vp, sp, vp, vp, sz, vp]
    L.usv_block_scores_static.restype, L.usv_block_scores_static.argtypes = i32, [vp, vp, sp, vp, vp]
    L.usv_select_topk.restype, L.usv_select_topk.argtypes = i32, [vp, sp, i32, vp, i32, vp, vp, vp]
    L.usv_select_topk_ex.restype = i32
    L.usv_select_topk_ex.argtypes = [vp, sp, i32, vp, i32, ctypes.c_uint32, vp, vp, vp]
    L.usv_coarse_workspace_bytes.restype, L.usv_coarse_workspace_bytes.argtypes = sz, [sp]
    L.usv_coarse_attn.restype, L.usv_coarse_attn.argtypes = i32, [vp, vp, sp, vp, vp, sz, vp]
    L.usv_fuse_outputs.restype, L.usv_fuse_outputs.argtypes = i32, [vp, i32, vp, vp, vp, sp, i32, vp, vp]
    L.usv_block_sparse_attn_fused.restype = i32
    L.usv_block_sparse_attn_fused.argtypes = [vp, vp, vp, sp, vp, vp, i32, f32, vp, vp, vp, i32, vp, vp, vp]
    L.usv_entropy_workspace_bytes.restype, L.usv_entropy_workspace_bytes.argtypes = sz, [sp]
    L.usv_attn_entropy.restype, L.usv_attn_entropy.argtypes = i32, [vp, sp, vp, vp, sz, vp]
    L.usv_entropy_allocate.restype = i32
    L.usv_entropy_allocate.argtypes = [vp, i32, f32, f32, f32, f32, vp]
    L.usv_block_sparse_attn.restype = i32
    L.usv_block_sparse_attn.argtypes = [vp, vp, vp, sp, vp, vp, i32, f32, i32, vp, vp, vp]
    L.usv_attn_work_order.restype, L.usv_attn_work_order.argtypes = i32, [vp, vp, sp, i32, vp, vp]
    L.usv_block_sparse_attn_ordered.restype = i32
    L.usv_block_sparse_attn_ordered.argtypes = [vp, vp, vp, sp, vp, vp, i32, vp, f32, i32, vp, vp, vp]
    gp, stp = ctypes.POINTER(UsvGrid), ctypes.POINTER(UsvStrides)
    L.usv_cube_token_order.restype, L.usv_cube_token_order.argtypes = i32, [gp, vp]
    L.usv_cube_gather.restype, L.usv_cube_gather.argtypes = i32, [vp, stp, sp, gp, vp, vp]
    L.usv_cube_scatter.restype, L.usv_cube_scatter.argtypes = i32, [vp, sp, gp, vp, stp, vp]
    L.usv_merge_workspace_bytes.restype, L.usv_merge_workspace_bytes.argtypes = sz, [sp, gp]
    L.usv_merge_similarity.restype, L.usv_merge_similarity.argtypes = i32, [vp, sp, gp, vp, vp, vp, sz, vp]
    L.usv_merge_plan.restype, L.usv_merge_plan.argtypes = i32, [vp, vp, sp, gp, vp, vp, vp, sz, vp]
    L.usv_merge_plan_workspace_bytes.restype, L.usv_merge_plan_workspace_bytes.argtypes = sz, [sp, gp]
    L.usv_merge_apply.restype, L.usv_merge_apply.argtypes = i32, [vp, sp, gp, vp, vp, vp, vp]
    L.usv_unmerge_apply.restype, L.usv_unmerge_apply.argtypes = i32, [vp, sp, gp, vp, vp, vp]
    rp = ctypes.POINTER(UsvRaster)
    L.usv_cube_order.restype, L.usv_cube_order.argtypes = i32, [sp, gp, vp, vp]
    L.usv_cube_count.restype, L.usv_cube_count.argtypes = i32, [gp]
    L.usv_cube_order_padded.restype, L.usv_cube_order_padded.argtypes = i32, [gp, vp, vp, vp]
    L.usv_block_scores_raster.restype, L.usv_block_scores_raster.argtypes = i32, [vp, vp, sp, rp, vp, vp, sz, vp]
    L.usv_block_sparse_attn_raster.restype = i32
    L.usv_block_sparse_attn_raster.argtypes = [vp, vp, vp, sp, rp, vp, vp, i32, f32, i32, vp, vp, vp]
    L.usv_coarse_attn_raster.restype, L.usv_coarse_attn_raster.argtypes = i32, [vp, vp, sp, rp, vp, vp, sz, vp]
    L.usv_block_sparse_attn_raster_fused.restype = i32
    L.usv_block_sparse_attn_raster_fused.argtypes = [vp, vp, vp, sp, rp, vp, vp, i32, f32, vp, vp, vp, i32, vp, vp, vp]
    L.usv_status_string.restype, L.usv_status_string.argtypes = ctypes.c_char_p, [i32]
    L.usv_last_error.restype, L.usv_last_error.argtypes = ctypes.c_char_p, []
    _lib = L
    return L


def _check(status: int):
    if status != 0:
        L = lib()
        raise UsvError(status, L.usv_status_string(status).decode(), L.usv_last_error().decode())


def _dev(t: torch.Tensor, name: str, dtype=None):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor (there is no CPU path)")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _shape_of(x: torch.Tensor, seq_valid) -> UsvShape:
    if x.dim() != 4:
        raise ValueError("Q/K/V must be [B, Hh, N, d]")
    if x.dtype == torch.bfloat16:
        dt = USV_BF16
    elif x.dtype == torch.float32:
        dt = USV_F32
    else:
        raise TypeError(f"unsupported dtype {x.dtype}")
    B, Hh, N, d = x.shape
    return UsvShape(B, Hh, N, N if seq_valid is None else int(seq_valid), d, BLOCK, dt)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def workspace_bytes(batch, heads, seq_len, seq_valid, head_dim, dtype) -> int:
    dt = USV_BF16 if dtype in (torch.bfloat16, "bf16") else USV_F32
    sh = UsvShape(batch, heads, seq_len, seq_valid, head_dim, BLOCK, dt)
    return int(lib().usv_workspace_bytes(ctypes.byref(sh)))


def block_scores(q, k, seq_valid=None, out=None, workspace=None):
    """usv_block_scores: pooled block scores [B, Hh, nb, nb] fp32 of Q, K [B, Hh, N, d]."""
    sh = _shape_of(q, seq_valid)
    if k.shape != q.shape or k.dtype != q.dtype:
        raise ValueError("k must match q in shape and dtype")
    nb = sh.seq_len // BLOCK
    if out is None:
        out = torch.empty((sh.batch, sh.heads, nb, nb), dtype=torch.float32, device=q.device)
    need = int(lib().usv_workspace_bytes(ctypes.byref(sh)))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(
        lib().usv_block_scores(
            _dev(q, "q"), _dev(k, "k"), ctypes.byref(sh), _dev(out, "scores", torch.float32),
            _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream(),
        )
    )
    return out


def block_scores_static(q, k, out, seq_valid=None):
    """usv_block_scores_static: stage 1 without a workspace; `out` [B, Hh, nb, nb] fp32 is the caller's."""
    sh = _shape_of(q, seq_valid)
    if k.shape != q.shape or k.dtype != q.dtype:
        raise ValueError("k must match q in shape and dtype")
    nb = sh.seq_len // BLOCK
    if tuple(out.shape) != (sh.batch, sh.heads, nb, nb):
        raise ValueError("out must be [B, Hh, nb, nb]")
    _check(lib().usv_block_scores_static(_dev(q, "q"), _dev(k, "k"), ctypes.byref(sh),
                                         _dev(out, "scores", torch.float32), _stream()))
    return out


TOPK_FORCE_LOCAL = 1


def select_topk(scores, k=0, seq_valid=None, budgets=None, kmax=None, idx=None, cnt=None, force_local=False):
    """usv_select_topk(_ex): scores [B, Hh, nb, nb] fp32 -> idx [B, Hh, nb, kmax] int32 (-1 padded), cnt [B, Hh, nb].

    force_local: USV_TOPK_FORCE_LOCAL, every row keeps its own cube."""
    if scores.dim() != 4 or scores.shape[2] != scores.shape[3]:
        raise ValueError("scores must be [B, Hh, nb, nb]")
    B, Hh, nb, _ = scores.shape
    N = nb * BLOCK
    sh = UsvShape(B, Hh, N, N if seq_valid is None else int(seq_valid), 0, BLOCK, USV_F32)
    if kmax is None:
        kmax = int(k)
    if idx is None:
        idx = torch.empty((B, Hh, nb, max(kmax, 1)), dtype=torch.int32, device=scores.device)
    if cnt is None:
        cnt = torch.empty((B, Hh, nb), dtype=torch.int32, device=scores.device)
    bptr = None if budgets is None else _dev(budgets, "budgets", torch.int32)
    args = (_dev(scores, "scores", torch.float32), ctypes.byref(sh), int(k), bptr, int(kmax))
    outs = (_dev(idx, "idx", torch.int32), _dev(cnt, "cnt", torch.int32), _stream())
    if force_local:
        _check(lib().usv_select_topk_ex(*args, TOPK_FORCE_LOCAL, *outs))
    else:
        _check(lib().usv_select_topk(*args, *outs))
    return idx, cnt


def attn_work_order(cnt, kmax, idx=None, out=None):
    """usv_attn_work_order: per head, the query blocks sorted by (list length descending, where the list lies
    [needs idx], block index) -> int32 [B, Hh, nb]."""
    B, Hh, nb = cnt.shape
    sh = UsvShape(B, Hh, nb * BLOCK, nb * BLOCK, 0, BLOCK, USV_F32)
    if out is None:
        out = torch.empty((B, Hh, nb), dtype=torch.int32, device=cnt.device)
    if idx is not None and (tuple(idx.shape[:3]) != (B, Hh, nb) or idx.shape[3] != kmax):
        raise ValueError("idx must be [B, Hh, nb, kmax]")
    _check(lib().usv_attn_work_order(None if idx is None else _dev(idx, "idx", torch.int32), _dev(cnt, "cnt", torch.int32),
                                     ctypes.byref(sh), int(kmax), _dev(out, "work_order", torch.int32), _stream()))
    return out


def block_sparse_attn(q, k, v, idx, cnt, seq_valid=None, scale=0.0, out=None, lse=None, return_lse=False,
                      out_dtype=None, coarse=None, gate_fine=None, gate_coarse=None, work_order=None):
    """usv_block_sparse_attn(_fused, _ordered): attention over the listed K/V blocks.  Returns out (and lse if asked).

    out_dtype: dtype of the result; defaults to q's dtype, torch.float32 is also allowed for bf16 inputs.
    coarse (+ optional gates): usv_block_sparse_attn_fused, out = gate_fine * attention + gate_coarse * coarse[cube].
    work_order (from attn_work_order): usv_block_sparse_attn_ordered, the launch walks the query blocks in that order."""
    sh = _shape_of(q, seq_valid)
    for name, t in (("k", k), ("v", v)):
        if t.shape != q.shape or t.dtype != q.dtype:
            raise ValueError(f"{name} must match q in shape and dtype")
    nb = sh.seq_len // BLOCK
    if idx.dim() != 4 or tuple(idx.shape[:3]) != (sh.batch, sh.heads, nb):
        raise ValueError("idx must be [B, Hh, nb, kmax]")
    if tuple(cnt.shape) != (sh.batch, sh.heads, nb):
        raise ValueError("cnt must be [B, Hh, nb]")
    kmax = idx.shape[3]
    if out is None:
        out = torch.empty_like(q, dtype=out_dtype or q.dtype)
    if out.shape != q.shape:
        raise ValueError("out must have q's shape")
    if out.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError(f"unsupported out dtype {out.dtype}")
    odt = USV_F32 if out.dtype == torch.float32 else USV_BF16
    if lse is None and return_lse:
        lse = torch.empty((sh.batch, sh.heads, sh.seq_len), dtype=torch.float32, device=q.device)
    head = (_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), ctypes.byref(sh), _dev(idx, "idx", torch.int32),
            _dev(cnt, "cnt", torch.int32), int(kmax), float(scale))
    tail = (odt, _dev(out, "out"), None if lse is None else _dev(lse, "lse", torch.float32), _stream())
    if work_order is not None:
        if coarse is not None or gate_fine is not None or gate_coarse is not None:
            raise ValueError("work_order and the fused second branch are separate calls")
        if tuple(work_order.shape) != (sh.batch, sh.heads, nb):
            raise ValueError("work_order must be [B, Hh, nb]")
        _check(lib().usv_block_sparse_attn_ordered(*head[:7], _dev(work_order, "work_order", torch.int32), head[7], *tail))
    elif coarse is None and gate_fine is None and gate_coarse is None:
        _check(lib().usv_block_sparse_attn(*head, *tail))
    else:
        for name, g in (("gate_fine", gate_fine), ("gate_coarse", gate_coarse)):
            if g is not None and (g.shape != q.shape or g.dtype != q.dtype):
                raise ValueError(f"{name} must match q in shape and dtype")
        _check(lib().usv_block_sparse_attn_fused(
            *head, None if coarse is None else _dev(coarse, "coarse", torch.float32),
            None if gate_fine is None else _dev(gate_fine, "gate_fine"),
            None if gate_coarse is None else _dev(gate_coarse, "gate_coarse"), *tail))
    return (out, lse) if return_lse else out


def _grid(grid, cube) -> UsvGrid:
    return UsvGrid(*(int(x) for x in grid), *(int(x) for x in cube))


def cube_token_order(grid, cube=(4, 4, 4)):
    """usv_cube_token_order (host): int32 array, order[p] = raster index of the token at cube-major position p."""
    import numpy as np

    g = _grid(grid, cube)
    order = np.full(max(int(grid[0]) * int(grid[1]) * int(grid[2]), 1), -1, dtype=np.int32)
    _check(lib().usv_cube_token_order(ctypes.byref(g), order.ctypes.data_as(ctypes.c_void_p)))
    return order


def _raster(t: torch.Tensor, name: str):
    """Pointer and element strides of a raster tensor [B, Hh, Nv, d] (any strides with the channel index contiguous)."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor (there is no CPU path)")
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError(f"{name} must be [B, Hh, Nv, d] with contiguous channels")
    return t.data_ptr(), UsvStrides(t.stride(0), t.stride(1), t.stride(2))


def cube_gather(raster, grid, cube=(4, 4, 4), seq_len=None, out=None):
    """usv_cube_gather: raster-ordered [B, Hh, T*H*W, d] (a strided view is fine) -> cube-major [B, Hh, seq_len, d]."""
    B, Hh, Nv, d = raster.shape
    if seq_len is None:
        seq_len = -(-Nv // BLOCK) * BLOCK
    if out is None:
        out = torch.empty((B, Hh, seq_len, d), dtype=raster.dtype, device=raster.device)
    if tuple(out.shape) != (B, Hh, seq_len, d) or out.dtype != raster.dtype:
        raise ValueError("out must be [B, Hh, seq_len, d] of the input dtype")
    sh = _shape_of(out, Nv)
    ptr, st = _raster(raster, "raster")
    g = _grid(grid, cube)
    _check(lib().usv_cube_gather(ptr, ctypes.byref(st), ctypes.byref(sh), ctypes.byref(g), _dev(out, "cube"), _stream()))
    return out


def cube_scatter(cube_major, grid, cube=(4, 4, 4), out=None):
    """usv_cube_scatter: cube-major [B, Hh, seq_len, d] -> raster order [B, Hh, T*H*W, d] (out may be a strided view)."""
    B, Hh, N, d = cube_major.shape
    Nv = int(grid[0]) * int(grid[1]) * int(grid[2])
    if out is None:
        out = torch.empty((B, Hh, Nv, d), dtype=cube_major.dtype, device=cube_major.device)
    if tuple(out.shape) != (B, Hh, Nv, d) or out.dtype != cube_major.dtype:
        raise ValueError("out must be [B, Hh, T*H*W, d] of the input dtype")
    sh = _shape_of(cube_major, Nv)
    ptr, st = _raster(out, "raster")
    g = _grid(grid, cube)
    _check(lib().usv_cube_scatter(_dev(cube_major, "cube"), ctypes.byref(sh), ctypes.byref(g), ptr, ctypes.byref(st), _stream()))
    return out


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return USV_F32
    if t.dtype == torch.bfloat16:
        return USV_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def coarse_attn(scores, v, seq_valid=None, out=None, workspace=None):
    """usv_coarse_attn: cube-level attention output [B, Hh, nb, d] fp32 from the block scores and V."""
    sh = _shape_of(v, seq_valid)
    nb = sh.seq_len // BLOCK
    if tuple(scores.shape) != (sh.batch, sh.heads, nb, nb):
        raise ValueError("scores must be [B, Hh, nb, nb]")
    if out is None:
        out = torch.empty((sh.batch, sh.heads, nb, sh.head_dim), dtype=torch.float32, device=v.device)
    need = int(lib().usv_coarse_workspace_bytes(ctypes.byref(sh)))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=v.device)
    _check(lib().usv_coarse_attn(_dev(scores, "scores", torch.float32), _dev(v, "v"), ctypes.byref(sh),
                                 _dev(out, "coarse", torch.float32), _dev(workspace, "workspace"),
                                 workspace.numel() * workspace.element_size(), _stream()))
    return out


def fuse_outputs(fine, coarse, gate_fine=None, gate_coarse=None, seq_valid=None, out=None, out_dtype=None):
    """usv_fuse_outputs: out = gate_fine * fine + gate_coarse * broadcast(coarse); gates None = 1."""
    B, Hh, N, d = fine.shape
    gates = [g for g in (gate_fine, gate_coarse) if g is not None]
    gdt = gates[0].dtype if gates else fine.dtype
    for g in gates:
        if g.shape != fine.shape or g.dtype != gdt:
            raise ValueError("gates must have fine's shape and one dtype")
    sh = UsvShape(B, Hh, N, N if seq_valid is None else int(seq_valid), d, BLOCK, USV_F32 if gdt == torch.float32 else USV_BF16)
    if tuple(coarse.shape) != (B, Hh, N // BLOCK, d):
        raise ValueError("coarse must be [B, Hh, nb, d]")
    if out is None:
        out = torch.empty_like(fine, dtype=out_dtype or fine.dtype)
    if out.shape != fine.shape:
        raise ValueError("out must have fine's shape")
    _check(lib().usv_fuse_outputs(_dev(fine, "fine"), _dt(fine), _dev(coarse, "coarse", torch.float32),
                                  None if gate_fine is None else _dev(gate_fine, "gate_fine"),
                                  None if gate_coarse is None else _dev(gate_coarse, "gate_coarse"),
                                  ctypes.byref(sh), _dt(out), _dev(out, "out"), _stream()))
    return out


def attn_entropy(scores, seq_valid=None, out=None, workspace=None):
    """usv_attn_entropy: normalised entropy [B] fp32 of the key marginal of the cube-level attention weights."""
    if scores.dim() != 4 or scores.shape[2] != scores.shape[3]:
        raise ValueError("scores must be [B, Hh, nb, nb]")
    B, Hh, nb, _ = scores.shape
    N = nb * BLOCK
    sh = UsvShape(B, Hh, N, N if seq_valid is None else int(seq_valid), 0, BLOCK, USV_F32)
    if out is None:
        out = torch.empty((B,), dtype=torch.float32, device=scores.device)
    need = int(lib().usv_entropy_workspace_bytes(ctypes.byref(sh)))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=scores.device)
    _check(lib().usv_attn_entropy(_dev(scores, "scores", torch.float32), ctypes.byref(sh), _dev(out, "entropy", torch.float32),
                                  _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()))
    return out


def entropy_allocate(entropy, rho_bar, gamma=1.0, rho_min=0.0, rho_max=1.0):
    """usv_entropy_allocate (host): per-layer sparsity ratios from per-layer entropies."""
    import numpy as np

    h = np.ascontiguousarray(np.asarray(entropy, dtype=np.float32).reshape(-1))
    rho = np.empty_like(h)
    _check(lib().usv_entropy_allocate(h.ctypes.data_as(ctypes.c_void_p), int(h.size), float(rho_bar), float(gamma),
                                      float(rho_min), float(rho_max), rho.ctypes.data_as(ctypes.c_void_p)))
    return rho


def _merge_shape(B, Hh, d, dtype, grid, r, seq_len=None) -> UsvShape:
    """Shape of the MERGED tensors: seq_valid = T*H*W - r rows, padded to seq_len (default: next multiple of 64)."""
    n_valid = int(grid[0]) * int(grid[1]) * int(grid[2]) - int(r)
    if seq_len is None:
        seq_len = -(-n_valid // BLOCK) * BLOCK
    return UsvShape(B, Hh, int(seq_len), n_valid, d, BLOCK, USV_BF16 if dtype == torch.bfloat16 else USV_F32)


def merge_similarity(k, grid, mblock, out=None, blk=None, workspace=None):
    """usv_merge_similarity: K [B, Hh, T*H*W, d] in raster order -> (u [B, T*H*W] fp32, -inf at destinations;
    blk [T*H*W] int32, the partition: block rank, bit 31 at destinations)."""
    B, Hh, N, d = k.shape
    sh = _merge_shape(B, Hh, d, k.dtype, grid, 0)
    g = _grid(grid, mblock)
    if out is None:
        out = torch.empty((B, N), dtype=torch.float32, device=k.device)
    if blk is None:
        blk = torch.empty((N,), dtype=torch.int32, device=k.device)
    need = int(lib().usv_merge_workspace_bytes(ctypes.byref(sh), ctypes.byref(g)))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=k.device)
    _check(lib().usv_merge_similarity(_dev(k, "k"), ctypes.byref(sh), ctypes.byref(g), _dev(out, "u", torch.float32),
                                      _dev(blk, "blk", torch.int32), _dev(workspace, "workspace"), workspace.numel(), _stream()))
    return out, blk


MERGE_PLAN_WIDE_TOKENS = 8192  # from here on merge_plan brings a workspace by itself: the selection runs chip-wide


def merge_plan_workspace_bytes(B, grid, mblock, r) -> int:
    sh = _merge_shape(B, 1, 64, torch.float32, grid, r)
    g = _grid(grid, mblock)
    return int(lib().usv_merge_plan_workspace_bytes(ctypes.byref(sh), ctypes.byref(g)))


def merge_plan(u, blk, grid, mblock, r, row_of=None, src_of=None, workspace=None):
    """usv_merge_plan: u [B, T*H*W] fp32 and the partition blk -> row_of [B, T*H*W], src_of [B, T*H*W - r] (int32).

    workspace: uint8 device tensor of merge_plan_workspace_bytes(...) -> the selection is spread over the chip; False ->
    one workgroup per batch element; None -> a workspace is allocated from MERGE_PLAN_WIDE_TOKENS tokens on."""
    B, N = u.shape
    sh = _merge_shape(B, 1, 64, torch.float32, grid, r)
    g = _grid(grid, mblock)
    if row_of is None:
        row_of = torch.empty((B, N), dtype=torch.int32, device=u.device)
    if src_of is None:
        src_of = torch.empty((B, max(N - int(r), 1)), dtype=torch.int32, device=u.device)[:, : N - int(r)]
    if workspace is None and N >= MERGE_PLAN_WIDE_TOKENS:
        workspace = torch.empty(int(lib().usv_merge_plan_workspace_bytes(ctypes.byref(sh), ctypes.byref(g))), dtype=torch.uint8,
                                device=u.device)
    if workspace is None or workspace is False:
        wptr, wbytes = None, 0
    else:
        wptr, wbytes = _dev(workspace, "workspace"), workspace.numel() * workspace.element_size()
    _check(lib().usv_merge_plan(_dev(u, "u", torch.float32), _dev(blk, "blk", torch.int32), ctypes.byref(sh), ctypes.byref(g),
                                _dev(row_of, "row_of", torch.int32), _dev(src_of, "src_of", torch.int32), wptr, wbytes, _stream()))
    return row_of, src_of


def merge_apply(x, grid, mblock, row_of, src_of, seq_len=None, out=None):
    """usv_merge_apply: raster x [B, Hh, T*H*W, d] -> merged [B, Hh, seq_len, d] (padding rows zero)."""
    B, Hh, N, d = x.shape
    sh = _merge_shape(B, Hh, d, x.dtype, grid, N - src_of.shape[1], seq_len)
    g = _grid(grid, mblock)
    if out is None:
        out = torch.empty((B, Hh, sh.seq_len, d), dtype=x.dtype, device=x.device)
    _check(lib().usv_merge_apply(_dev(x, "x"), ctypes.byref(sh), ctypes.byref(g), _dev(row_of, "row_of", torch.int32),
                                 _dev(src_of, "src_of", torch.int32), _dev(out, "out"), _stream()))
    return out


def unmerge_apply(y, grid, mblock, row_of, n_merged_rows, out=None):
    """usv_unmerge_apply: merged y [B, Hh, seq_len, d] (n_merged_rows real rows) -> raster [B, Hh, T*H*W, d]."""
    B, Hh, Np, d = y.shape
    N = row_of.shape[1]
    sh = _merge_shape(B, Hh, d, y.dtype, grid, N - int(n_merged_rows), Np)
    g = _grid(grid, mblock)
    if out is None:
        out = torch.empty((B, Hh, N, d), dtype=y.dtype, device=y.device)
    _check(lib().usv_unmerge_apply(_dev(y, "y"), ctypes.byref(sh), ctypes.byref(g), _dev(row_of, "row_of", torch.int32),
                                   _dev(out, "out"), _stream()))
    return out


def cube_order(grid, cube=(4, 4, 4), seq_len=None, device="cuda:0", out=None):
    """usv_cube_order: the order table on the device, int32 [seq_len] (padding positions hold 0)."""
    Nv = int(grid[0]) * int(grid[1]) * int(grid[2])
    if seq_len is None:
        seq_len = -(-Nv // BLOCK) * BLOCK
    if out is None:
        out = torch.empty((seq_len,), dtype=torch.int32, device=device)
    sh = UsvShape(1, 1, int(seq_len), Nv, 0, BLOCK, USV_F32)
    g = _grid(grid, cube)
    _check(lib().usv_cube_order(ctypes.byref(sh), ctypes.byref(g), _dev(out, "order", torch.int32), _stream()))
    return out


def cube_order_padded(grid, cube=(4, 4, 4), device="cuda:0"):
    """usv_cube_order_padded: one cube per block, cut cubes padded -> (order int32 [64 * cubes], block_valid int32 [cubes])."""
    g = _grid(grid, cube)
    n = int(lib().usv_cube_count(ctypes.byref(g)))
    if n == 0:
        raise ValueError("invalid grid / cube, or too many cubes")
    order = torch.empty((n * BLOCK,), dtype=torch.int32, device=device)
    valid = torch.empty((n,), dtype=torch.int32, device=device)
    _check(lib().usv_cube_order_padded(ctypes.byref(g), _dev(order, "order", torch.int32),
                                       _dev(valid, "block_valid", torch.int32), _stream()))
    return order, valid


def _view(order, st, ost, block_valid, work_order=None):
    bv = None
    if block_valid is not None:
        if block_valid.numel() * BLOCK != order.numel():
            raise ValueError("block_valid must hold one count per 64 entries of order")
        bv = _dev(block_valid, "block_valid", torch.int32)
    wo = None if work_order is None else _dev(work_order, "work_order", torch.int32)
    return UsvRaster(_dev(order, "order", torch.int32), st, ost, bv, wo)


def _raster_shape(x, order):
    B, Hh, Nv, d = x.shape
    return UsvShape(B, Hh, order.numel(), Nv, d, BLOCK, USV_BF16 if x.dtype == torch.bfloat16 else USV_F32)


def block_scores_raster(q, k, order, out=None, workspace=None, block_valid=None):
    """usv_block_scores_raster: q, k raster-ordered [B, Hh, Nv, d] (strided views allowed) -> scores [B, Hh, nb, nb].

    block_valid (with the order table of cube_order_padded): one cube per block, cut cubes padded."""
    sh = _raster_shape(q, order)
    qp, st = _raster(q, "q")
    kp, st_k = _raster(k, "k")
    if (st_k.batch, st_k.head, st_k.token) != (st.batch, st.head, st.token) or k.dtype != q.dtype:
        raise ValueError("k must match q in strides and dtype")
    nb = sh.seq_len // BLOCK
    if out is None:
        out = torch.empty((sh.batch, sh.heads, nb, nb), dtype=torch.float32, device=q.device)
    need = int(lib().usv_workspace_bytes(ctypes.byref(sh)))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    view = _view(order, st, UsvStrides(0, 0, 0), block_valid)
    _check(lib().usv_block_scores_raster(qp, kp, ctypes.byref(sh), ctypes.byref(view), _dev(out, "scores", torch.float32),
                                         _dev(workspace, "workspace"), workspace.numel(), _stream()))
    return out


def coarse_attn_raster(scores, v, order, out=None, workspace=None, block_valid=None):
    """usv_coarse_attn_raster: usv_coarse_attn with v in raster order [B, Hh, Nv, d] (strided views allowed)."""
    sh = _raster_shape(v, order)
    vp_, st = _raster(v, "v")
    nb = sh.seq_len // BLOCK
    if tuple(scores.shape) != (sh.batch, sh.heads, nb, nb):
        raise ValueError("scores must be [B, Hh, nb, nb]")
    if out is None:
        out = torch.empty((sh.batch, sh.heads, nb, sh.head_dim), dtype=torch.float32, device=v.device)
    need = int(lib().usv_coarse_workspace_bytes(ctypes.byref(sh)))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=v.device)
    view = _view(order, st, UsvStrides(0, 0, 0), block_valid)
    _check(lib().usv_coarse_attn_raster(_dev(scores, "scores", torch.float32), vp_, ctypes.byref(sh), ctypes.byref(view),
                                        _dev(out, "coarse", torch.float32), _dev(workspace, "workspace"),
                                        workspace.numel() * workspace.element_size(), _stream()))
    return out


def block_sparse_attn_raster(q, k, v, order, idx, cnt, scale=0.0, out=None, out_dtype=None, return_lse=False,
                             coarse=None, gate_fine=None, gate_coarse=None, block_valid=None, work_order=None):
    """usv_block_sparse_attn_raster(_fused): raster-ordered q, k, v [B, Hh, Nv, d] -> out [B, Hh, Nv, d] in raster order.

    coarse (+ optional raster-order gates laid out like q): out = gate_fine * attention + gate_coarse * coarse[cube]."""
    sh = _raster_shape(q, order)
    ptrs = []
    st = None
    for name, t in (("q", q), ("k", k), ("v", v)):
        p, s_t = _raster(t, name)
        if st is None:
            st = s_t
        elif (s_t.batch, s_t.head, s_t.token) != (st.batch, st.head, st.token) or t.dtype != q.dtype:
            raise ValueError(f"{name} must match q in strides and dtype")
        ptrs.append(p)
    if out is None:
        out = torch.empty(q.shape, dtype=out_dtype or q.dtype, device=q.device)
    op, ost = _raster(out, "out")
    lse = torch.empty((sh.batch, sh.heads, sh.seq_valid), dtype=torch.float32, device=q.device) if return_lse else None
    if work_order is not None and tuple(work_order.shape) != (sh.batch, sh.heads, sh.seq_len // BLOCK):
        raise ValueError("work_order must be [B, Hh, nb]")
    view = _view(order, st, ost, block_valid, work_order)
    gates = []
    for name, g_ in (("gate_fine", gate_fine), ("gate_coarse", gate_coarse)):
        if g_ is None:
            gates.append(None)
            continue
        gp_, gst = _raster(g_, name)
        if (gst.batch, gst.head, gst.token) != (st.batch, st.head, st.token) or g_.dtype != q.dtype or g_.shape != q.shape:
            raise ValueError(f"{name} must match q in shape, strides and dtype")
        gates.append(gp_)
    _check(lib().usv_block_sparse_attn_raster_fused(
        *ptrs, ctypes.byref(sh), ctypes.byref(view), _dev(idx, "idx", torch.int32), _dev(cnt, "cnt", torch.int32),
        int(idx.shape[3]), float(scale), None if coarse is None else _dev(coarse, "coarse", torch.float32), gates[0],
        gates[1], _dt(out), op, None if lse is None else _dev(lse, "lse", torch.float32), _stream()))
    return (out, lse) if return_lse else out
