"""The three stages driven from plain C (paper_2512_05754_amd/tools/usv_demo.c: C99, the C ABI and the HIP runtime, no
Python in the process) against the oracle: scores at the fp32 bound, selection bit-exact on the program's own scores,
attention at the bf16 bound."""
import os
import subprocess

import numpy as np
import pytest

import gpu_util as gu
from oracle import usv_oracle as orc
from paper_2512_05754_amd import synth
from paper_2512_05754_amd.build import DEMO_TOOL

pytestmark = pytest.mark.gpu


def test_three_stages_from_a_c_program(tmp_path):
    if not os.path.exists(DEMO_TOOL):  # a host program (gcc, seconds): built here if the tree came without it
        from paper_2512_05754_amd import binding
        from paper_2512_05754_amd.build import build_demo

        binding.lib()
        build_demo(verbose=False)
    w = synth.Workload("c_demo", 2, 3, 11 * 64 - 17, 128, "bf16", 2.0, 4, seed=7301)
    Q, K, V = synth.gen_qkv(w)
    for name, x in (("q", Q), ("k", K), ("v", V)):
        x.tofile(tmp_path / f"{name}.bin")
    (tmp_path / "shape.txt").write_text(f"{w.batch} {w.heads} {w.seq_len} {w.seq_valid} {w.head_dim} {w.keep}\n")
    res = subprocess.run([DEMO_TOOL, str(tmp_path)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    B, Hh, N, d, nb, k = w.batch, w.heads, w.seq_len, w.head_dim, w.nb, w.keep
    S = np.fromfile(tmp_path / "scores.bin", dtype=np.float32).reshape(B, Hh, nb, nb)
    idx = np.fromfile(tmp_path / "idx.bin", dtype=np.int32).reshape(B, Hh, nb, k)
    cnt = np.fromfile(tmp_path / "cnt.bin", dtype=np.int32).reshape(B, Hh, nb)
    out = np.fromfile(tmp_path / "out.bin", dtype=np.float32).reshape(B, Hh, N, d)
    Qf, Kf, Vf = synth.as_f32(Q), synth.as_f32(K), synth.as_f32(V)
    gu.assert_f32_close(S, orc.block_scores(Qf, Kf, w.seq_valid), "scores from C")
    ridx, rcnt = orc.select_topk(S, k, w.seq_valid)
    np.testing.assert_array_equal(idx, ridx)
    np.testing.assert_array_equal(cnt, rcnt)
    ref = orc.block_sparse_attn(Qf.astype(np.float64), Kf.astype(np.float64), Vf.astype(np.float64), ridx, rcnt, w.seq_valid)[0]
    gu.assert_attn_close(out[:, :, :w.seq_valid], ref[:, :, :w.seq_valid], "bf16", "attention from C")
