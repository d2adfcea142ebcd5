"""Seeded synthetic Q/K/V generators shaped like the video-DiT attention workloads.

This module only draws random numbers and packs them into the storage formats
the attention path consumes (fp32, or bf16 bit patterns in uint16).  It holds
none of the method's arithmetic: no pooling, scoring, selection or softmax.
Both the CPU oracle's tests and the HIP path's tests/bench take inputs from
here so that the two sides always see the same bits.

Recipe (per (batch, head) pair, so any head can be regenerated on its own):
    rng   = numpy.random.default_rng([seed, b, h])
    draws = noise_Q, noise_K, noise_V  (each [N, d], i.i.d. N(0,1), fp32)
            u_Q, u_K, u_V              (each [nb, d], i.i.d. N(0,1), fp32)
    X     = noise_X + cube_gain * repeat(u_X, 64 rows per block)
The shared per-block vector u stands for the spatial/temporal redundancy inside
one 4x4x4 cube of video-latent tokens and makes the pooled block scores
strongly non-uniform (std about cube_gain^2), so that top-k selection is a
meaningful, data-dependent choice.  Rows r >= seq_valid (padding up to a
multiple of the block size) are overwritten with a finite sentinel so that a
kernel that leaks padded keys or queries into the result is caught.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

BLOCK = 64
PAD_SENTINEL = 1000.0  # finite, bf16-exact, far outside the bulk of N(0,1)+2u


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    heads: int
    seq_valid: int  # Nv: real tokens (T*H*W of the latent grid, after merging)
    head_dim: int
    dtype: str  # "f32" or "bf16"
    cube_gain: float  # 0 => plain N(0,1)
    keep: int  # uniform budget k (blocks kept per query block); 0 => ragged
    budget_lo: int = 0
    budget_hi: int = 0
    seed: int = 20251205

    @property
    def seq_len(self) -> int:  # N: padded to a multiple of the block size
        return (self.seq_valid + BLOCK - 1) // BLOCK * BLOCK

    @property
    def nb(self) -> int:
        return self.seq_len // BLOCK

    @property
    def kmax(self) -> int:
        return self.keep if self.keep else self.budget_hi


def keep_count(keep_ratio: float, nb: int) -> int:
    """Blocks kept for a keep ratio: floor, at least one."""
    return max(1, int(np.floor(keep_ratio * nb + 1e-9)))


# The five workloads the benchmark contract names.
TINY = Workload("tiny_4x16x16_f32", 1, 2, 4 * 16 * 16, 64, "f32", 0.0, 4, seed=20251205)
WAN13_480P = Workload("wan1.3b_480p_keep10", 1, 12, 21 * 30 * 52, 128, "bf16", 2.0, 51, seed=20251206)
WAN14_720P = Workload("wan14b_720p_keep5", 1, 40, 21 * 45 * 80, 128, "bf16", 2.0, 59, seed=20251208)
MERGED_RAGGED = Workload(
    "merged_480p_ragged", 2, 12, 16384, 128, "bf16", 2.0, 0, budget_lo=8, budget_hi=64, seed=20251209
)


def sweep(keep_ratio: float) -> Workload:
    k = keep_count(keep_ratio, WAN13_480P.nb)
    return replace(WAN13_480P, name=f"wan1.3b_480p_keep{int(round(keep_ratio * 100))}", keep=k, seed=20251207)


SWEEP_RATIOS = (1.0, 0.5, 0.25, 0.10, 0.05)


# --------------------------------------------------------------------------- #
# bf16 storage helpers (format conversion only)
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- #
# generators
# --------------------------------------------------------------------------- #
def gen_head_f32(w: Workload, b: int, h: int):
    """Q, K, V of one (batch, head) as fp32 arrays [N, d] (before any bf16 rounding)."""
    N, d, nb = w.seq_len, w.head_dim, w.nb
    rng = np.random.default_rng([w.seed, b, h])
    noise = [rng.standard_normal((N, d), dtype=np.float32) for _ in range(3)]
    cube = [rng.standard_normal((nb, d), dtype=np.float32) for _ in range(3)]
    out = []
    for n, u in zip(noise, cube):
        if w.cube_gain != 0.0:
            n += np.float32(w.cube_gain) * np.repeat(u, BLOCK, axis=0)
        n[w.seq_valid:] = PAD_SENTINEL
        out.append(n)
    return out


def gen_head(w: Workload, b: int, h: int):
    """Q, K, V of one (batch, head) in storage format: fp32, or uint16 bf16 bits."""
    q, k, v = gen_head_f32(w, b, h)
    if w.dtype == "bf16":
        return f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v)
    return q, k, v


def gen_qkv(w: Workload):
    """Full Q, K, V [B, Hh, N, d] in storage format (contiguous, d innermost)."""
    st = np.uint16 if w.dtype == "bf16" else np.float32
    shape = (w.batch, w.heads, w.seq_len, w.head_dim)
    Q, K, V = (np.empty(shape, dtype=st) for _ in range(3))
    for b in range(w.batch):
        for h in range(w.heads):
            Q[b, h], K[b, h], V[b, h] = gen_head(w, b, h)
    return Q, K, V


def gen_budgets(w: Workload) -> np.ndarray:
    """Per-(batch, head, query block) key budgets, int32 [B, Hh, nb], uniform in [lo, hi]."""
    rng = np.random.default_rng([w.seed, 0xB0D6E7])
    return rng.integers(w.budget_lo, w.budget_hi + 1, size=(w.batch, w.heads, w.nb), dtype=np.int32)


def as_f32(x: np.ndarray) -> np.ndarray:
    """Storage format -> fp32 values (exact)."""
    return bf16_bits_to_f32(x) if x.dtype == np.uint16 else np.asarray(x, dtype=np.float32)


def gen_raster_qkv(w: Workload, grid, cube):
    """Q, K, V [B, Hh, T*H*W, d] in RASTER token order, storage format, with the shared vector u drawn per TRUE
    cube of the grid (cubes cut by the boundary included): X = noise + cube_gain * u[cube of the token].
    w.seq_valid must be T*H*W; the draws are rng([seed, b, h]): noise_Q, noise_K, noise_V, u_Q, u_K, u_V."""
    T, H, Wd = grid
    ct, ch, cw = cube
    n = T * H * Wd
    assert w.seq_valid == n
    nH, nW = -(-H // ch), -(-Wd // cw)
    t, h, x = np.meshgrid(np.arange(T), np.arange(H), np.arange(Wd), indexing="ij")
    cube_of = (((t // ct) * nH + h // ch) * nW + x // cw).reshape(-1)
    n_cubes = -(-T // ct) * nH * nW
    st = np.uint16 if w.dtype == "bf16" else np.float32
    out = [np.empty((w.batch, w.heads, n, w.head_dim), dtype=st) for _ in range(3)]
    for b in range(w.batch):
        for hd in range(w.heads):
            rng = np.random.default_rng([w.seed, b, hd])
            noise = [rng.standard_normal((n, w.head_dim), dtype=np.float32) for _ in range(3)]
            us = [rng.standard_normal((n_cubes, w.head_dim), dtype=np.float32) for _ in range(3)]
            for o, nz, u in zip(out, noise, us):
                val = nz + np.float32(w.cube_gain) * u[cube_of]
                o[b, hd] = f32_to_bf16_bits(val) if w.dtype == "bf16" else val
    return out
