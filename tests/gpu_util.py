"""Helpers shared by the GPU parity tests (upload/download and the acceptance bounds)."""
import numpy as np
import torch

from oracle import usv_oracle as orc
from paper_2512_05754_amd import synth

DEV = "cuda:0"

# Acceptance bounds.
#  fp32 inputs: 1e-5 relative, taken as |delta| <= 1e-5 * max(1, |ref|) elementwise (scores and attention).
#  bf16 inputs: scores as above (the pooled sums are fp32 sums of values that are exact in fp32);
#               attention output max-abs <= 2e-2 and mean-abs <= 2e-3 on the fp32-stored result; a
#               bf16-stored result must be, bit for bit, that fp32 result rounded to nearest even
#               (assert_bf16_store_is_rne): the one extra rounding is then the only thing that sets it apart.
F32_REL = 1e-5
BF16_MAX_ABS = 2e-2
BF16_MEAN_ABS = 2e-3


def up(x: np.ndarray) -> torch.Tensor:
    """Storage-format numpy array (fp32, int32 or uint16 bf16 bits) -> GPU tensor."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def down(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


def assert_f32_close(got, ref, what=""):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    same_inf = np.isinf(ref) & (got == ref)
    bound = F32_REL * np.maximum(1.0, np.abs(np.where(np.isinf(ref), 0.0, ref)))
    bad = ~same_inf & ~(np.abs(got - np.where(np.isinf(ref), np.nan, ref)) <= bound)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} beyond 1e-5 relative; worst {np.nanmax(np.abs(got - ref)[bad]):.3e}"


def assert_attn_close(got, ref, in_dtype, what=""):
    """fp32-stored attention output against the oracle: the bounds above, nothing added."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    if in_dtype == "f32":
        assert_f32_close(got, ref, what)
        return err.max(), err.mean()
    assert (err <= BF16_MAX_ABS).all(), f"{what}: max-abs {err.max():.3e} beyond {BF16_MAX_ABS}"
    assert err.mean() <= BF16_MEAN_ABS, f"{what}: mean-abs {err.mean():.3e} > {BF16_MEAN_ABS}"
    return err.max(), err.mean()


def assert_bf16_store_is_rne(out_bf16: torch.Tensor, out_f32: torch.Tensor, what=""):
    """The bf16-stored output is the fp32-stored one (same launch shape, same accumulators) rounded once,
    to nearest even: compared as bit patterns, every element."""
    assert out_bf16.dtype == torch.bfloat16 and out_f32.dtype == torch.float32 and out_bf16.shape == out_f32.shape
    want = out_f32.to(torch.bfloat16).view(torch.int16)
    same = out_bf16.view(torch.int16) == want
    assert bool(same.all()), f"{what}: {int((~same).sum())} of {same.numel()} elements are not RNE(fp32 result)"


def oracle_attn_blocks(Qh, Kh, Vh, idx_h, cnt_h, seq_valid, qblocks, scale=None):
    """Oracle rows of the listed query blocks of one head: returns {i: (O[64,d], lse[64])}."""
    O, lse = orc.block_sparse_attn_head(synth.as_f32(Qh), synth.as_f32(Kh), synth.as_f32(Vh), idx_h, cnt_h,
                                        seq_valid, scale, qblocks)
    return {i: (O[i * 64:(i + 1) * 64], lse[i * 64:(i + 1) * 64]) for i in qblocks}
