"""GPU parity tests: every stage of the HIP path, through the C ABI binding, against the CPU oracle on the
same seeded inputs.  Sizes here are ones the oracle finishes in seconds and that still span several
tiles and a ragged tail; the full benchmark shapes are in test_gpu_fullsize.py."""
import numpy as np
import pytest
import torch

import gpu_util as gu
from oracle import usv_oracle as orc
from paper_2512_05754_amd import synth
from paper_2512_05754_amd.synth import Workload

pytestmark = pytest.mark.gpu


def small_workloads():
    return [
        synth.TINY,
        Workload("f32_d128_ragged", 1, 2, 5 * 64 - 17, 128, "f32", 2.0, 2, seed=11),
        Workload("bf16_d128_ragged", 2, 3, 9 * 64 - 9, 128, "bf16", 2.0, 4, seed=12),
        Workload("bf16_d64", 1, 2, 6 * 64, 64, "bf16", 2.0, 3, seed=13),
        Workload("bf16_d64_ragged", 1, 1, 6 * 64 - 40, 64, "bf16", 1.0, 5, seed=14),
        Workload("bf16_d128_70blocks", 1, 1, 70 * 64 - 1, 128, "bf16", 2.0, 7, seed=15),
        Workload("f32_d128_64blocks", 1, 2, 64 * 64 - 7, 128, "f32", 2.0, 8, seed=16),
        Workload("f32_d64_40blocks", 1, 1, 40 * 64 - 33, 64, "f32", 2.0, 6, seed=17),
    ]


@pytest.mark.parametrize("w", small_workloads(), ids=lambda w: w.name)
def test_block_scores(usv, w):
    Q, K, _ = synth.gen_qkv(w)
    S = usv.block_scores(gu.up(Q), gu.up(K), seq_valid=w.seq_valid)
    ref = orc.block_scores(synth.as_f32(Q), synth.as_f32(K), w.seq_valid)
    gu.assert_f32_close(gu.down(S), ref, w.name)


def test_block_scores_fully_padded_blocks(usv):
    w = Workload("pad2", 1, 1, 3 * 64 + 5, 64, "bf16", 2.0, 1, seed=3)
    Q, K, _ = synth.gen_qkv(w)
    # give the call two extra, fully padded blocks
    pad = np.full((1, 1, 128, 64), synth.f32_to_bf16_bits(np.float32(synth.PAD_SENTINEL)), dtype=np.uint16)
    Q, K = np.concatenate([Q, pad], axis=2), np.concatenate([K, pad], axis=2)
    S = gu.down(usv.block_scores(gu.up(Q), gu.up(K), seq_valid=w.seq_valid))
    ref = orc.block_scores(synth.as_f32(Q), synth.as_f32(K), w.seq_valid)
    assert np.isneginf(S[0, 0, 4:, :]).all() and np.isneginf(S[0, 0, :, 4:]).all()
    gu.assert_f32_close(S, ref)


# --------------------------------------------------------------------------- #
def check_topk(usv, S, k, seq_valid, budgets=None, kmax=None):
    idx, cnt = usv.select_topk(gu.up(S), k=k, seq_valid=seq_valid,
                               budgets=None if budgets is None else gu.up(budgets), kmax=kmax)
    ridx, rcnt = orc.select_topk(S, k, seq_valid, budgets=budgets, kmax=kmax)
    assert np.array_equal(gu.down(cnt), rcnt)
    assert np.array_equal(gu.down(idx), ridx)  # bit-exact, including the -1 padding


@pytest.mark.parametrize("nb,k", [(16, 4), (16, 1), (16, 16), (64, 7), (65, 64), (100, 37), (512, 51), (512, 512),
                                  (512, 256), (1182, 59), (300, 1)])
def test_topk_random(usv, nb, k):
    rng = np.random.default_rng(nb * 1000 + k)
    rows = 2 if nb > 600 else 3
    S = rng.standard_normal((1, rows, nb, nb)).astype(np.float32) * 4
    check_topk(usv, S, k, nb * 64)


def test_topk_ties_and_special_values(usv):
    nb = 128
    rng = np.random.default_rng(5)
    S = np.round(rng.standard_normal((1, 2, nb, nb)) * 2).astype(np.float32)  # heavy duplicates
    S[0, 0, 0, :] = 0.0  # all equal
    S[0, 0, 1, :] = np.where(rng.random(nb) < 0.5, -0.0, 0.0)  # signed zeros
    S[0, 0, 2, ::3] = -np.inf
    S[0, 0, 3, ::2] = np.nan
    S[0, 0, 4, :] = np.nan
    S[0, 0, 5, :] = -np.inf
    S[0, 0, 6, :] = np.inf
    S[0, 0, 7, :] = np.concatenate([np.full(nb - 3, np.nan), [-np.inf, 1.0, np.nan]])
    S[0, 0, 8, :] = np.float32(1e-40) * rng.integers(-3, 4, nb)  # denormals around zero
    for k in (1, 2, 40, 64, 127, 128):
        check_topk(usv, S, k, nb * 64)
    check_topk(usv, S, 40, nb * 64 - 64 * 3 - 5)  # only 125 candidate blocks, partial last one


@pytest.mark.parametrize("force_local", [False, True], ids=["plain", "force_local"])
def test_topk_adversarial_rows(usv, force_local):
    """Rows built to stress the threshold search: huge dynamic range, values one ulp apart, a single
    outlier, all negative, few distinct values, signalling NaNs, infinities at the local cube."""
    nb = 192  # three register slots per lane, the last rows only partly valid below
    rng = np.random.default_rng(77)
    S = np.empty((1, 1, nb, nb), dtype=np.float32)
    base = rng.standard_normal((nb, nb)).astype(np.float32)
    for i in range(nb):
        kind = i % 12
        r = base[i].copy()
        if kind == 0:
            r = np.exp(rng.uniform(-80, 80, nb)).astype(np.float32) * rng.choice([-1, 1], nb)  # 2^-115 .. 2^115
        elif kind == 1:
            r = (np.float32(3.0) + np.arange(nb, dtype=np.float32) * np.float32(2.0 ** -22))[rng.permutation(nb)]
        elif kind == 2:
            r[:] = -5.0
            r[rng.integers(nb)] = 1e30
        elif kind == 3:
            r = -np.abs(r) - 1  # no positive score in the row
        elif kind == 4:
            r = rng.integers(0, 3, nb).astype(np.float32)  # three distinct values
        elif kind == 5:
            r.view(np.uint32)[::5] = 0x7FA00000  # signalling NaNs, positive
            r.view(np.uint32)[1::7] = 0xFFA00001  # and negative ones
        elif kind == 6:
            r[i] = np.inf  # the local cube ties with other +inf scores
            r[::9] = np.inf
        elif kind == 7:
            r[i] = np.nan  # the local cube has no score at all
        elif kind == 8:
            r[i] = -np.inf
            r[1::2] = -np.inf
        elif kind == 9:
            r = (rng.integers(-4, 5, nb) * np.float32(1e-41)).astype(np.float32)  # denormals and zeros of both signs
            r[::4] *= np.float32(-1.0)
        elif kind == 10:
            r[:] = np.float32(np.finfo(np.float32).max)
            r[::2] = -np.float32(np.finfo(np.float32).max)
        S[0, 0, i] = r
    for seq_valid in (nb * 64, nb * 64 - 64 * 60 - 3):
        for k in (1, 2, 17, 64, 65, 130, nb):
            idx, cnt = usv.select_topk(gu.up(S), k=k, seq_valid=seq_valid, force_local=force_local)
            ridx, rcnt = orc.select_topk(S, k, seq_valid, force_local=force_local)
            assert np.array_equal(gu.down(cnt), rcnt), (seq_valid, k)
            assert np.array_equal(gu.down(idx), ridx), (seq_valid, k)


def test_topk_ragged_budgets(usv):
    nb, kmax = 256, 64
    rng = np.random.default_rng(9)
    S = rng.standard_normal((2, 2, nb, nb)).astype(np.float32)
    budgets = rng.integers(8, 65, size=(2, 2, nb), dtype=np.int32)
    budgets[0, 0, :6] = [0, -3, 1, 64, 65, 1000]
    check_topk(usv, S, 0, nb * 64, budgets=budgets, kmax=kmax)
    check_topk(usv, S, 0, nb * 64 - 100, budgets=budgets, kmax=kmax)


# --------------------------------------------------------------------------- #
def run_pipeline(usv, w, out_dtype=None, budgets=None):
    Q, K, V = synth.gen_qkv(w)
    q, k, v = gu.up(Q), gu.up(K), gu.up(V)
    S = usv.block_scores(q, k, seq_valid=w.seq_valid)
    idx, cnt = usv.select_topk(S, k=w.keep, seq_valid=w.seq_valid, kmax=w.kmax,
                               budgets=None if budgets is None else gu.up(budgets))
    out, lse = usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, return_lse=True, out_dtype=out_dtype)
    torch.cuda.synchronize()
    return (Q, K, V), gu.down(S), gu.down(idx), gu.down(cnt), out, gu.down(lse)


@pytest.mark.parametrize("w", small_workloads(), ids=lambda w: w.name)
def test_pipeline_against_oracle(usv, w):
    """scores -> top-k -> attention; the oracle selects from the SAME fp32 scores the GPU produced."""
    (Q, K, V), S, idx, cnt, out, lse = run_pipeline(usv, w, out_dtype=torch.float32)
    ridx, rcnt = orc.select_topk(S, w.keep, w.seq_valid)
    assert np.array_equal(idx, ridx) and np.array_equal(cnt, rcnt)
    O, L = orc.block_sparse_attn(synth.as_f32(Q), synth.as_f32(K), synth.as_f32(V), ridx, rcnt, w.seq_valid)
    gu.assert_attn_close(gu.down(out), O, w.dtype, w.name)
    live = np.isfinite(L)
    assert np.array_equal(np.isneginf(lse), ~live)
    assert np.abs(lse[live] - L[live]).max() <= (1e-4 if w.dtype == "f32" else 2e-2)
    assert (gu.down(out)[..., w.seq_valid:, :] == 0).all()


DEGENERATE = [
    Workload("one_token_bf16", 1, 1, 1, 128, "bf16", 2.0, 1, seed=31),        # a single valid token in a single block
    Workload("one_token_f32", 2, 1, 1, 64, "f32", 0.0, 1, seed=32),
    Workload("block_plus_one_bf16", 1, 2, 65, 64, "bf16", 2.0, 2, seed=33),   # second block holds one token
    Workload("block_plus_one_f32", 1, 1, 65, 128, "f32", 2.0, 1, seed=34),
    Workload("one_block_exact_bf16", 1, 1, 64, 128, "bf16", 2.0, 1, seed=35),  # no padding at all, one tile
]


@pytest.mark.parametrize("w", DEGENERATE, ids=lambda w: w.name)
def test_degenerate_sizes_against_oracle(usv, w):
    """The smallest shapes the ABI admits: one token, one block, a block with a single valid token."""
    (Q, K, V), S, idx, cnt, out, lse = run_pipeline(usv, w, out_dtype=torch.float32)
    Qf, Kf, Vf = (synth.as_f32(x) for x in (Q, K, V))
    gu.assert_f32_close(S, orc.block_scores(Qf, Kf, w.seq_valid), w.name + " scores")
    ridx, rcnt = orc.select_topk(S, w.keep, w.seq_valid)
    assert np.array_equal(idx, ridx) and np.array_equal(cnt, rcnt)
    O, L = orc.block_sparse_attn(Qf, Kf, Vf, ridx, rcnt, w.seq_valid)
    gu.assert_attn_close(gu.down(out), O, w.dtype, w.name)
    live = np.isfinite(L)
    assert np.array_equal(np.isneginf(lse), ~live)
    assert np.abs(lse[live] - L[live]).max() <= (1e-4 if w.dtype == "f32" else 2e-2)
    if w.seq_valid == 1:  # softmax over one key: the output row is that key's value row
        np.testing.assert_allclose(gu.down(out)[:, :, 0], Vf[:, :, 0], rtol=0, atol=1e-6)


@pytest.mark.parametrize("w", [x for x in small_workloads() if x.dtype == "bf16"] +
                         [x for x in DEGENERATE if x.dtype == "bf16"], ids=lambda w: w.name)
def test_bf16_output_storage(usv, w):
    """Output stored in the input dtype: bit for bit the fp32-stored result rounded to nearest even, every element;
    the fp32-stored result is the one held to the 2e-2 / 2e-3 bounds against the oracle."""
    (Q, K, V), S, idx, cnt, out, lse = run_pipeline(usv, w)
    assert out.dtype == torch.bfloat16
    _, S32, idx32, cnt32, out32, lse32 = run_pipeline(usv, w, out_dtype=torch.float32)
    assert np.array_equal(idx, idx32) and np.array_equal(cnt, cnt32)
    gu.assert_bf16_store_is_rne(out, out32, w.name)
    np.testing.assert_array_equal(lse, lse32)
    O, _ = orc.block_sparse_attn(synth.as_f32(Q), synth.as_f32(K), synth.as_f32(V), idx, cnt, w.seq_valid)
    gu.assert_attn_close(gu.down(out32), O, w.dtype, w.name)


def arbitrary_lists(w, rng, kmax):
    nbv = (w.seq_valid + 63) // 64
    idx = np.full((w.batch, w.heads, w.nb, kmax), -1, dtype=np.int32)
    cnt = np.zeros((w.batch, w.heads, w.nb), dtype=np.int32)
    for b in range(w.batch):
        for h in range(w.heads):
            for i in range(w.nb):
                c = int(rng.integers(0, min(kmax, nbv) + 1))
                idx[b, h, i, :c] = rng.choice(nbv, size=c, replace=False)  # unsorted on purpose
                cnt[b, h, i] = c
    return idx, cnt


@pytest.mark.parametrize("w", [small_workloads()[1], small_workloads()[2], small_workloads()[4]], ids=lambda w: w.name)
def test_attention_with_arbitrary_lists(usv, w):
    """Static / caller-made lists: unsorted, ragged, some empty, some holding only the partial block."""
    rng = np.random.default_rng(21)
    Q, K, V = synth.gen_qkv(w)
    idx, cnt = arbitrary_lists(w, rng, 5)
    nbv = (w.seq_valid + 63) // 64
    idx[0, 0, 0, 0], cnt[0, 0, 0] = nbv - 1, 1  # only the partial block
    cnt[0, 0, 1] = 0
    out, lse = usv.block_sparse_attn(gu.up(Q), gu.up(K), gu.up(V), gu.up(idx), gu.up(cnt), seq_valid=w.seq_valid,
                                     return_lse=True, out_dtype=torch.float32)
    O, L = orc.block_sparse_attn(synth.as_f32(Q), synth.as_f32(K), synth.as_f32(V), idx, cnt, w.seq_valid)
    gu.assert_attn_close(gu.down(out), O, w.dtype, w.name)
    assert (gu.down(out)[0, 0, 64:128] == 0).all() and np.isneginf(gu.down(lse)[0, 0, 64:128]).all()
    # a custom softmax scale
    out2 = usv.block_sparse_attn(gu.up(Q), gu.up(K), gu.up(V), gu.up(idx), gu.up(cnt), seq_valid=w.seq_valid,
                                 scale=0.05, out_dtype=torch.float32)
    O2, _ = orc.block_sparse_attn(synth.as_f32(Q), synth.as_f32(K), synth.as_f32(V), idx, cnt, w.seq_valid, scale=0.05)
    gu.assert_attn_close(gu.down(out2), O2, w.dtype, w.name + " scale")


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128)])
def test_lists_naming_wholly_padded_blocks(usv, dtype, d):
    """Tensors padded by whole blocks (seq_valid several blocks short of seq_len) and caller-made lists that name
    the padded blocks too: their keys are all masked (the mask of the masked-attention equation is 0 for them),
    so they add nothing, and a row whose list holds nothing else is an empty row (0, lse = -inf)."""
    nb, Nv = 8, 5 * 64 - 20  # blocks 0..3 whole, 4 partial, 5..7 padding only
    w = Workload("whole_block_padding", 1, 2, nb * 64, d, dtype, 2.0, 4, seed=77)
    Q, K, V = synth.gen_qkv(w)
    for x in (Q, K, V):
        x[:, :, Nv:] = synth.f32_to_bf16_bits(np.float32(synth.PAD_SENTINEL)) if dtype == "bf16" else synth.PAD_SENTINEL
    kmax = 6
    idx = np.full((1, 2, nb, kmax), -1, dtype=np.int32)
    cnt = np.zeros((1, 2, nb), dtype=np.int32)
    rows = [[5], [7, 6], [0, 5, 3], [6, 4], [4, 7], [1, 2, 5, 6, 7, 0], [5, 6, 7], [2]]
    for h in range(2):
        for i, r in enumerate(rows):
            r = r if h == 0 else r[::-1]
            idx[0, h, i, :len(r)], cnt[0, h, i] = r, len(r)
    out, lse = usv.block_sparse_attn(gu.up(Q), gu.up(K), gu.up(V), gu.up(idx), gu.up(cnt), seq_valid=Nv,
                                     return_lse=True, out_dtype=torch.float32)
    O, L = orc.block_sparse_attn(synth.as_f32(Q), synth.as_f32(K), synth.as_f32(V), idx, cnt, Nv)
    got, got_lse = gu.down(out), gu.down(lse)
    gu.assert_attn_close(got, O, dtype, "whole-block padding")
    live = np.isfinite(L)
    assert np.array_equal(np.isneginf(got_lse), ~live)
    assert np.abs(got_lse[live] - L[live]).max() <= (1e-4 if dtype == "f32" else 2e-2)
    for i in (0, 1, 6):  # lists of padded blocks only
        assert not got[0, :, i * 64:(i + 1) * 64].any() and np.isneginf(got_lse[0, :, i * 64:(i + 1) * 64]).all()


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64)])
def test_keep_all_equals_dense_attention(usv, dtype, d):
    w = Workload("dense", 1, 2, 6 * 64 - 5, d, dtype, 1.0, 6, seed=31)
    Q, K, V = synth.gen_qkv(w)
    idx = np.tile(np.arange(6, dtype=np.int32), (1, 2, 6, 1))
    cnt = np.full((1, 2, 6), 6, dtype=np.int32)
    out = usv.block_sparse_attn(gu.up(Q), gu.up(K), gu.up(V), gu.up(idx), gu.up(cnt), seq_valid=w.seq_valid,
                                out_dtype=torch.float32)
    Nv = w.seq_valid
    for h in range(2):
        q, k, v = (synth.as_f32(x[0, h, :Nv]) for x in (Q, K, V))
        O, _ = orc.dense_attn(q, k, v)
        gu.assert_attn_close(gu.down(out)[0, h, :Nv], O, dtype, "dense")


@pytest.mark.parametrize("nb,k", [(200, 70), (200, 67), (140, 100), (130, 129), (330, 64), (330, 65)])
def test_long_lists_cross_the_index_reload_boundary(usv, nb, k):
    """Lists longer than 64 entries (the kernel keeps 64 block ids in a register and reloads), in both
    launch shapes (k < nb/2: deep ring; k >= nb/2: three workgroups per CU), with a padded last block."""
    w = Workload(f"long_{nb}_{k}", 1, 1, nb * 64 - 11, 128, "bf16", 2.0, k, seed=71 + nb + k)
    (Q, K, V), S, idx, cnt, out, lse = run_pipeline(usv, w, out_dtype=torch.float32)
    ridx, rcnt = orc.select_topk(S, w.keep, w.seq_valid)
    assert np.array_equal(idx, ridx) and np.array_equal(cnt, rcnt)
    blocks = [0, 1, nb // 2, nb - 2, nb - 1]
    ref = gu.oracle_attn_blocks(Q[0, 0], K[0, 0], V[0, 0], ridx[0, 0], rcnt[0, 0], w.seq_valid, blocks)
    got = np.stack([gu.down(out[0, 0, i * 64:(i + 1) * 64]) for i in blocks])
    gu.assert_attn_close(got, np.stack([ref[i][0] for i in blocks]), "bf16", w.name)


@pytest.mark.parametrize("nb,kmax,d", [(64, 24, 128), (64, 24, 64), (24, 24, 128), (40, 40, 64)],
                         ids=["sparse_shape_d128", "sparse_shape_d64", "dense_shape_d128", "dense_shape_d64"])
def test_every_list_length_in_both_launch_shapes(usv, nb, kmax, d):
    """Query cube i gets a list of i % (kmax + 1) blocks: every length from 0 to kmax, i.e. every phase of the
    K/V ring and every shape of its last, partial round, in the sparse launch shape (kmax < nb/2: five slots)
    and in the dense-like one (three slots)."""
    w = Workload("lengths", 1, 2, nb * 64 - 11, d, "bf16", 2.0, kmax, seed=300 + nb + d)
    rng = np.random.default_rng(nb * 7 + kmax + d)
    Q, K, V = synth.gen_qkv(w)
    nbv = (w.seq_valid + 63) // 64
    idx = np.full((1, 2, nb, kmax), -1, dtype=np.int32)
    cnt = np.zeros((1, 2, nb), dtype=np.int32)
    for h in range(2):
        for i in range(nb):
            c = (i + 3 * h) % (kmax + 1)
            idx[0, h, i, :c] = np.sort(rng.choice(nbv, size=c, replace=False))
            cnt[0, h, i] = c
    out, lse = usv.block_sparse_attn(gu.up(Q), gu.up(K), gu.up(V), gu.up(idx), gu.up(cnt), seq_valid=w.seq_valid,
                                     return_lse=True, out_dtype=torch.float32)
    O, L = orc.block_sparse_attn(synth.as_f32(Q), synth.as_f32(K), synth.as_f32(V), idx, cnt, w.seq_valid)
    gu.assert_attn_close(gu.down(out), O, "bf16", f"nb {nb} kmax {kmax}")
    live = np.isfinite(L)
    assert np.array_equal(np.isneginf(gu.down(lse)), ~live)
    assert np.abs(gu.down(lse)[live] - L[live]).max() <= 2e-2


def test_online_softmax_survives_large_logit_offsets(usv):
    """Keys shifted by a large common vector: every logit of a row moves by the same amount."""
    w = Workload("shift", 1, 1, 8 * 64, 128, "bf16", 0.0, 8, seed=41)
    Q, K, V = synth.gen_qkv(w)
    Kf = synth.as_f32(K) + np.float32(6.0)  # logits shift by 6*sum(q)/sqrt(d): tens to hundreds
    K = synth.f32_to_bf16_bits(Kf)
    idx = np.tile(np.arange(8, dtype=np.int32)[::-1], (1, 1, 8, 1)).copy()
    cnt = np.full((1, 1, 8), 8, dtype=np.int32)
    out = usv.block_sparse_attn(gu.up(Q), gu.up(K), gu.up(V), gu.up(idx), gu.up(cnt), out_dtype=torch.float32)
    O, _ = orc.block_sparse_attn(synth.as_f32(Q), synth.as_f32(K), synth.as_f32(V), idx, cnt, w.seq_valid)
    gu.assert_attn_close(gu.down(out), O, "bf16", "shift")


def test_rows_sum_to_one_and_determinism(usv):
    w = Workload("ones", 1, 2, 10 * 64 - 3, 128, "bf16", 2.0, 4, seed=51)
    Q, K, V = synth.gen_qkv(w)
    V1 = np.full_like(V, synth.f32_to_bf16_bits(np.float32(1.0)))
    q, k = gu.up(Q), gu.up(K)
    S = usv.block_scores(q, k, seq_valid=w.seq_valid)
    idx, cnt = usv.select_topk(S, k=4, seq_valid=w.seq_valid)
    out = gu.down(usv.block_sparse_attn(q, k, gu.up(V1), idx, cnt, seq_valid=w.seq_valid, out_dtype=torch.float32))
    np.testing.assert_allclose(out[..., : w.seq_valid, :], 1.0, rtol=0, atol=1e-5)
    a = usv.block_sparse_attn(q, k, gu.up(V), idx, cnt, seq_valid=w.seq_valid)
    b = usv.block_sparse_attn(q, k, gu.up(V), idx, cnt, seq_valid=w.seq_valid)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    S2 = usv.block_scores(q, k, seq_valid=w.seq_valid)
    assert torch.equal(S, S2)


@pytest.mark.parametrize("w", [small_workloads()[1], small_workloads()[2]], ids=lambda w: w.name)
def test_bad_list_contents_are_clamped_not_followed(usv, w):
    """The kernels clamp block ids into [0, nb) and counts into [0, kmax] before they become addresses: rows
    with a damaged list hold unspecified (finite or not) values, every other row is exactly what it was."""
    rng = np.random.default_rng(23)
    Q, K, V = synth.gen_qkv(w)
    idx, cnt = arbitrary_lists(w, rng, 4)
    q, k, v = gu.up(Q), gu.up(K), gu.up(V)
    good = usv.block_sparse_attn(q, k, v, gu.up(idx), gu.up(cnt), seq_valid=w.seq_valid, out_dtype=torch.float32)
    bad_idx, bad_cnt = idx.copy(), cnt.copy()
    bad_idx[0, 0, 0, :] = [-7, w.nb, 1 << 30, -(1 << 31)][:bad_idx.shape[3]]   # ids far outside the tensors
    bad_cnt[0, 0, 0] = bad_idx.shape[3]
    bad_cnt[0, 1, 1] = bad_idx.shape[3] + 1000                                   # count beyond the row stride
    bad_cnt[0, 1, 2] = -5
    out = usv.block_sparse_attn(q, k, v, gu.up(bad_idx), gu.up(bad_cnt), seq_valid=w.seq_valid, out_dtype=torch.float32)
    torch.cuda.synchronize()
    keep = torch.ones(good.shape[:3], dtype=torch.bool, device=good.device)
    keep[0, 0, 0:64] = False
    keep[0, 1, 64:192] = False
    assert torch.equal(out[keep], good[keep])
    assert (out[0, 1, 128:192] == 0).all()  # a negative count is an empty list


def test_outputs_do_not_spill_past_their_buffers(usv):
    """Canaries around scores, idx and out stay intact."""
    w = Workload("canary", 1, 2, 5 * 64 - 1, 128, "bf16", 2.0, 3, seed=61)
    Q, K, V = synth.gen_qkv(w)
    q, k, v = gu.up(Q), gu.up(K), gu.up(V)
    nb = w.nb

    def guarded(numel, dtype, fill):
        buf = torch.full((numel + 512,), fill, dtype=dtype, device=gu.DEV)
        return buf, buf[256:256 + numel]

    sbuf, s = guarded(2 * nb * nb, torch.float32, 777.0)
    ibuf, ix = guarded(2 * nb * 3, torch.int32, 777)
    cbuf, ct = guarded(2 * nb, torch.int32, 777)
    obuf, o = guarded(q.numel(), torch.float32, 777.0)
    S = usv.block_scores(q, k, seq_valid=w.seq_valid, out=s.view(1, 2, nb, nb))
    idx, cnt = usv.select_topk(S, k=3, seq_valid=w.seq_valid, idx=ix.view(1, 2, nb, 3), cnt=ct.view(1, 2, nb))
    usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, out=o.view(q.shape))
    torch.cuda.synchronize()
    for buf in (sbuf, ibuf, cbuf, obuf):
        assert (buf[:256] == 777).all() and (buf[-256:] == 777).all()
    assert not (o == 777).any()


def test_errors_surface_as_exceptions(usv):
    x = torch.zeros(1, 1, 128, 64, device=gu.DEV)
    with pytest.raises(usv.UsvError, match="USV_ERR_INVALID_ARG"):
        usv.select_topk(torch.zeros(1, 1, 2, 2, device=gu.DEV), k=3)
    with pytest.raises(usv.UsvError, match="USV_ERR_UNSUPPORTED"):
        usv.block_scores(torch.zeros(1, 1, 128, 96, device=gu.DEV), torch.zeros(1, 1, 128, 96, device=gu.DEV))
    with pytest.raises(usv.UsvError, match="USV_ERR_WORKSPACE"):
        usv.block_scores(x, x, workspace=torch.zeros(16, dtype=torch.uint8, device=gu.DEV))


def test_three_stages_replay_from_a_hip_graph(usv):
    """The calls only enqueue kernels on the caller's stream (no allocation, no memset, no host sync), so a
    serving loop can capture them once and replay: every replay, with eager work and synchronisation in
    between and fresh data in the captured buffers, must equal the eager result bit for bit."""
    w = Workload("graph", 1, 2, 7 * 64 - 3, 128, "bf16", 2.0, 3, seed=71)
    nb = w.nb
    q, k, v = (torch.empty((1, 2, w.seq_len, 128), dtype=torch.bfloat16, device=gu.DEV) for _ in range(3))
    S = torch.empty((1, 2, nb, nb), dtype=torch.float32, device=gu.DEV)
    ws = torch.empty(usv.workspace_bytes(1, 2, w.seq_len, w.seq_valid, 128, "bf16"), dtype=torch.uint8, device=gu.DEV)
    idx = torch.empty((1, 2, nb, 3), dtype=torch.int32, device=gu.DEV)
    cnt = torch.empty((1, 2, nb), dtype=torch.int32, device=gu.DEV)
    out = torch.empty((1, 2, w.seq_len, 128), dtype=torch.float32, device=gu.DEV)

    def step():
        usv.block_scores(q, k, seq_valid=w.seq_valid, out=S, workspace=ws)
        usv.select_topk(S, k=3, seq_valid=w.seq_valid, idx=idx, cnt=cnt)
        usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, out=out)

    def load(seed):
        Q, K, V = synth.gen_qkv(Workload("graph", 1, 2, w.seq_valid, 128, "bf16", 2.0, 3, seed=seed))
        for dst, src in ((q, Q), (k, K), (v, V)):
            dst.copy_(gu.up(src))

    load(71)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up on the capture stream, as torch asks for
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for seed in (72, 73, 74):
        load(seed)
        step()                       # eager
        torch.cuda.synchronize()
        want = (S.clone(), idx.clone(), cnt.clone(), out.clone())
        for t in (S, idx, cnt, out):
            t.fill_(7)               # eager work between the replays; also proves the replay writes everything
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((S, idx, cnt, out), want):
            assert torch.equal(got.view(torch.int32), ref.view(torch.int32))


# --------------------------------------------------------------------------- #
# longest-list-first work order
# --------------------------------------------------------------------------- #
def expected_work_order(idx, cnt, kmax):
    """The documented key, on the host: (kmax - len, buckets of the entries at 1/4, 1/2, 3/4 of the list, block index)."""
    B, Hh, nb = cnt.shape
    out = np.empty((B, Hh, nb), dtype=np.int32)
    for b in range(B):
        for h in range(Hh):
            c = np.clip(cnt[b, h], 0, kmax).astype(np.int64)
            pos = np.zeros(nb, dtype=np.int64)
            if idx is not None:
                for quarter in (1, 2, 3):
                    e = np.maximum(c - 1, 0) * quarter // 4
                    j = np.clip(idx[b, h, np.arange(nb), e], 0, nb - 1).astype(np.int64)
                    pos = (pos << 6) | np.where(c > 0, j * 64 // nb, 0)
                pos = np.where(c > 0, pos, 0)
            key = ((kmax - c) << 30) | (pos << 12) | np.arange(nb)
            out[b, h] = np.argsort(key, kind="stable")
    return out


def test_work_order_is_the_documented_sort_and_does_not_change_the_result(usv):
    """usv_attn_work_order: per head the query blocks sorted by (list length descending, where the list lies, index);
    usv_block_sparse_attn_ordered: the same bits as usv_block_sparse_attn whatever permutation it is given."""
    w = Workload("ragged_small", 2, 3, 40 * 64 - 17, 128, "bf16", 2.0, 0, budget_lo=0, budget_hi=24, seed=77)
    Q, K, V = synth.gen_qkv(w)
    q, k, v = gu.up(Q), gu.up(K), gu.up(V)
    budgets = synth.gen_budgets(w)
    budgets[0, 0, :5] = [0, 24, 24, 1, 0]
    S = usv.block_scores(q, k, seq_valid=w.seq_valid)
    idx, cnt = usv.select_topk(S, seq_valid=w.seq_valid, budgets=gu.up(budgets), kmax=w.kmax)
    i_h, c_h = gu.down(idx), gu.down(cnt)
    order = usv.attn_work_order(cnt, w.kmax, idx=idx)
    o_h = gu.down(order)
    np.testing.assert_array_equal(o_h, expected_work_order(i_h, c_h, w.kmax))
    np.testing.assert_array_equal(gu.down(usv.attn_work_order(cnt, w.kmax)), expected_work_order(None, c_h, w.kmax))
    for b in range(w.batch):
        for h in range(w.heads):
            assert sorted(o_h[b, h].tolist()) == list(range(w.nb))
            assert (np.diff(c_h[b, h][o_h[b, h]]) <= 0).all()
    ref, lse_ref = usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, out_dtype=torch.float32, return_lse=True)
    rng = np.random.default_rng(3)
    shuffled = np.stack([np.stack([rng.permutation(w.nb) for _ in range(w.heads)]) for _ in range(w.batch)]).astype(np.int32)
    for wo in (order, gu.up(shuffled), gu.up(np.ascontiguousarray(o_h[..., ::-1]))):
        out, lse = usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, out_dtype=torch.float32, return_lse=True,
                                         work_order=wo)
        assert torch.equal(out.view(torch.int32), ref.view(torch.int32))
        assert torch.equal(lse.view(torch.int32), lse_ref.view(torch.int32))
    # and the ordered call against the oracle
    O, _ = orc.block_sparse_attn(synth.as_f32(Q), synth.as_f32(K), synth.as_f32(V), i_h, c_h, w.seq_valid)
    gu.assert_attn_close(gu.down(ref), O, "bf16", "ragged lists")


@pytest.mark.parametrize("nb,kmax", [(700, 700), (1, 1), (2, 1), (64, 7), (1182, 59), (4096, 16)])
def test_work_order_sizes(usv, nb, kmax):
    """Block counts that are no power of two (the sort pads), one block, the largest supported count, kmax = nb."""
    rng = np.random.default_rng(5 + nb)
    B, Hh = 1, 2
    cnt = rng.integers(0, kmax + 1, size=(B, Hh, nb), dtype=np.int32)
    idx = np.full((B, Hh, nb, kmax), -1, dtype=np.int32)
    for h in range(Hh):
        for i in range(nb):
            idx[0, h, i, :cnt[0, h, i]] = np.sort(rng.choice(nb, size=cnt[0, h, i], replace=False))
    cnt[0, 0, :2] = [kmax, 0][:min(2, nb)]
    idx[0, 0, 0, :kmax] = np.sort(rng.choice(nb, size=kmax, replace=False))
    order = gu.down(usv.attn_work_order(gu.up(cnt), kmax, idx=gu.up(idx)))
    np.testing.assert_array_equal(order, expected_work_order(idx, cnt, kmax))
