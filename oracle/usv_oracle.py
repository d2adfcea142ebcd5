"""CPU fp64 oracle for dynamic block-sparse video attention.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the HIP kernels are compared against.  It is not a
product path: only tests, the smoke check and the benchmark's CPU-baseline leg
may import it, and it shares no code with the HIP path.  Everything is plain
NumPy in float64, written so it can be checked against the paper by eye; no
tiling, no online softmax, no fusion.

What it computes (paper: Section 3.2 "Video Sparse Attention", the unnumbered
dense-attention and masked-attention equations; Section 2.2's coarse-to-fine
description; Figure 2's "top-k cube selection"):

  1. block_scores   coarse stage: one score per (query cube, key cube) pair from
                    the mean-pooled query and key of each 64-token cube.
  2. select_topk    per query cube, the k best-scoring key cubes -> index list.
  3. block_sparse_attn
                    softmax((Q K^T + log M) / sqrt(d_k)) V with the 0/1 mask M
                    being block-structured: M[r, c] = 1 iff cube(c) is in the
                    list of cube(r).  Entries with log M = -inf contribute
                    exp(-inf) = 0, so only the listed cubes' keys are summed.
  masked_dense_attn the same equation written with the full N x N mask, for
                    small N (pins the gathered form above).
  dense_attn        softmax(Q K^T / sqrt(d_k)) V, the keep-all limit.

  cube_token_order / cube_gather / cube_scatter
                    the step either side of the path (Figure 2, right: the tokens are
                    split into small 3-D cubes on the way in, and the results are
                    spread over the whole token grid again on the way out): the permutation
                    between raster (t, h, w) token order and cube-major order.

  coarse_attn / fuse_outputs
                    the cube-level branch and the fusion of Figure 2 (right), for which the
                    paper prints no formula: the readings below.

  attention_entropy / entropy_allocate
                    Section 3.4 ("Entropy-aware dynamic sparsification policy"): the
                    key marginal of the attention weights averaged over heads and
                    queries, its normalised entropy, the weight (1 - h)^gamma and the
                    clipped, mean-preserving redistribution of a base sparsity.

  merge_plan / merge_apply / unmerge_apply
                    Section 3.3 ("Token merging for video"): 3-D bipartite partition,
                    head-averaged key descriptors, cosine similarity, the r most
                    confident sources, mean aggregation into the destinations, the
                    merged sequence [unmerged sources || destinations], and the
                    exact unmerge.

Every function is pinned by tests/test_oracle_pins.py against something other
than itself (closed forms, torch's scaled_dot_product_attention in fp64,
pure-Python brute force, invariants).  No function here is "parity unpinned".

Readings taken where the paper is silent:
  * score = mean(Q_cube) . mean(K_cube) / sqrt(d); means over valid tokens only;
    a cube with no valid token scores -inf; result rounded once to fp32.
  * selection is per (batch, head, query cube); candidates are the cubes that
    hold at least one valid token; order = (score descending, index ascending)
    on canonical values (-0 == +0, NaN below -inf); the list is emitted in
    ascending cube index, unused slots hold -1.
  * log M is added to the scaled logit (it is 0 or -inf, so where the division
    by sqrt(d_k) is drawn makes no difference).
  * cube-major order of a T x H x W grid tiled by ct x ch x cw cubes: cubes that
    lie wholly inside the grid come first, in raster order of their cube
    coordinates, one per 64-token block; the cubes cut by the grid boundary
    follow in the same raster order, packed without gaps (so only the tail of
    the sequence is padding, which is what seq_valid expresses); inside a cube,
    tokens are in raster order of their local coordinates.
  * cube-faithful variant of that order (cube_token_order_padded): every cube, cut or not, gets a 64-position
    block of its own, in raster order of the cube coordinates; a cut cube's tokens come first in its block and
    the rest of the block is padding.  The stages then take per-block valid counts (block_valid) in place of
    the single seq_valid: means over a block's valid tokens, padded keys masked, padded query rows 0.
  * coarse branch (the cube level of the coarse-to-fine scheme, Section 2.2): attention
    among the pooled cubes, C_i = sum_j softmax_j(S_ij) mean(V_j) over the cubes that hold
    a valid token, with S the stage-1 scores (they already carry the 1/sqrt(d)).
  * fusion (Figure 2 only says that the branch outputs are spread over the token grid and combined): every token r of cube i
    receives C_i; out_r = g_fine[r] * O_fine[r] + g_coarse[r] * C_cube(r), elementwise, with
    per-token, per-channel gates supplied by the model (absent gate = 1).
  * attention entropy: the paper takes the marginal of the full N x N attention weights,
    which a sparse kernel never forms (and does not say how it obtains them); here the
    weights are the cube-level ones, A[h,i,:] = softmax_j(S[h,i,:]) over the cubes with a
    valid token, and N in the equations is the number of such cubes.  With one token per
    cube this is the paper's definition exactly.  0 log 0 = 0; one cube gives h = 0.
  * token merging: tokens are in raster order of the T x H x W grid; the merge blocks
    (s_t, s_h, s_w) tile the grid from the origin and are cut by its boundary; the
    destination of a block is its first token (local coordinates 0,0,0), every other token
    of the block is a source.  Section 3.3 confines sources and destinations to the same local 3-D
    block: the only candidate destination of a source is the one of its own block, so j*(i) is that
    token and u_i their cosine similarity (a zero descriptor gives similarity 0).  The r
    selected sources are the first r in the order (u descending, raster index ascending);
    on canonical values as in the top-k selection (-0 equals +0, NaN ranks lowest); the merged
    sequence lists the unmerged sources, then the destinations, each in ascending raster index.
  * padded keys (token >= seq_valid) are masked; padded query rows output 0 and
    lse = -inf; a query cube with an empty list outputs 0.
"""
from __future__ import annotations

import math

import numpy as np

BLOCK = 64


def _f64(x):
    return np.asarray(x, dtype=np.float64)


# --------------------------------------------------------------------------- #
# stage 1: pooled block scores (coarse stage of the coarse-to-fine scheme)
# --------------------------------------------------------------------------- #
def _valid_counts(nb, seq_valid, block, block_valid):
    """Valid tokens of each block: block_valid[i] if given (the first block_valid[i] rows of block i), else the
    blocks are filled front to back by the first seq_valid tokens."""
    if block_valid is not None:
        v = np.asarray(block_valid, dtype=np.int64)
        assert v.shape == (nb,) and (v >= 0).all() and (v <= block).all()
        return v
    return np.clip(seq_valid - block * np.arange(nb), 0, block)


def block_means(X, seq_valid, block=BLOCK, block_valid=None):
    """Mean over the valid tokens of each block.  X: [..., N, d] -> [..., nb, d] (fp64).

    Blocks without a valid token get NaN means (they have no mean)."""
    X = _f64(X)
    N, d = X.shape[-2], X.shape[-1]
    nb = N // block
    nv = _valid_counts(nb, seq_valid, block, block_valid)
    out = np.full(X.shape[:-2] + (nb, d), np.nan)
    for i in range(nb):
        if nv[i] > 0:
            out[..., i, :] = X[..., i * block : i * block + nv[i], :].sum(axis=-2) / nv[i]
    return out


def block_scores(Q, K, seq_valid, block=BLOCK, block_valid=None):
    """S[b,h,i,j] = mean(Q_blk i) . mean(K_blk j) / sqrt(d), fp64 then rounded once to fp32.

    Q, K: [B, Hh, N, d].  Rows/columns of blocks with no valid token are -inf.
    block_valid: per-block valid counts (one cube per block, cut cubes padded: cube_token_order_padded)."""
    d = Q.shape[-1]
    qm = block_means(Q, seq_valid, block, block_valid)
    km = block_means(K, seq_valid, block, block_valid)
    nb = qm.shape[-2]
    live = _valid_counts(nb, seq_valid, block, block_valid) > 0
    S = np.full(qm.shape[:-2] + (nb, nb), -np.inf)
    ii = np.nonzero(live)[0]
    S[np.ix_(*[np.arange(n) for n in S.shape[:-2]], ii, ii)] = (
        np.einsum("...id,...jd->...ij", qm[..., ii, :], km[..., ii, :]) / math.sqrt(d)
    )
    return S.astype(np.float32)


# --------------------------------------------------------------------------- #
# stage 2: top-k key-block selection
# --------------------------------------------------------------------------- #
def select_topk_row(scores_row, k, nb_valid):
    """Indices of the k best of scores_row[:nb_valid], ascending; ties -> lower index."""
    s = np.asarray(scores_row[:nb_valid], dtype=np.float32)
    isnan = np.isnan(s)
    canon = np.where(isnan, -np.inf, s).astype(np.float64) + 0.0  # -0 -> +0
    # primary: score descending; then NaN after every number (also after -inf); then index ascending
    order = np.lexsort((np.arange(nb_valid), isnan, -canon))
    keep = order[: max(0, min(int(k), nb_valid))]
    return np.sort(keep).astype(np.int32)


def select_topk(S, k, seq_valid, budgets=None, kmax=None, block=BLOCK, force_local=False):
    """S: fp32 [B, Hh, nb, nb].  Returns idx int32 [B,Hh,nb,kmax] (-1 padded) and cnt int32 [B,Hh,nb].

    A row keeps min(budget, kmax, nb_valid) blocks where budget = budgets[b,h,i] if given else k.
    Query blocks with no valid token keep nothing.
    force_local (Figure 2, right: part of the budget goes to attention inside the local cube): a row that
    keeps anything keeps its own cube i, and fills the rest of its budget with the best OTHER cubes."""
    B, Hh, nb, _ = S.shape
    nb_valid = (seq_valid + block - 1) // block
    if kmax is None:
        kmax = int(k)
    idx = np.full((B, Hh, nb, kmax), -1, dtype=np.int32)
    cnt = np.zeros((B, Hh, nb), dtype=np.int32)
    for b in range(B):
        for h in range(Hh):
            for i in range(nb_valid):
                want = int(budgets[b, h, i]) if budgets is not None else int(k)
                want = max(0, min(want, kmax))
                if force_local and want >= 1:
                    others = np.array([j for j in range(nb_valid) if j != i], dtype=np.int64)
                    best = select_topk_row(S[b, h, i][others], want - 1, len(others))
                    sel = np.sort(np.concatenate([others[best], [i]])).astype(np.int32)
                else:
                    sel = select_topk_row(S[b, h, i], want, nb_valid)
                idx[b, h, i, : len(sel)] = sel
                cnt[b, h, i] = len(sel)
    return idx, cnt


# --------------------------------------------------------------------------- #
# stage 3: attention
# --------------------------------------------------------------------------- #
def _softmax_rows(L):
    """Row softmax and log-sum-exp of a logit matrix that may hold -inf entries."""
    m = L.max(axis=-1, keepdims=True)
    e = np.exp(L - m)
    z = e.sum(axis=-1, keepdims=True)
    return e / z, (m + np.log(z))[..., 0]


def dense_attn(Q, K, V, scale=None):
    """softmax(Q K^T / sqrt(d_k)) V for one head.  Q,K,V: [N, d].  (Dense-attention equation, Sec. 3.2.)"""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    scale = 1.0 / math.sqrt(Q.shape[-1]) if scale is None else scale
    P, lse = _softmax_rows((Q @ K.T) * scale)
    return P @ V, lse


def masked_dense_attn(Q, K, V, M, scale=None):
    """softmax(Q K^T / sqrt(d_k) + log M) V for one head, M a full N x N 0/1 mask.  (Masked equation, Sec. 3.2.)

    Every row of M must allow at least one key."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    scale = 1.0 / math.sqrt(Q.shape[-1]) if scale is None else scale
    with np.errstate(divide="ignore"):
        logM = np.log(_f64(M))
    P, lse = _softmax_rows((Q @ K.T) * scale + logM)
    return P @ V, lse


def block_mask(idx, cnt, seq_len, seq_valid, block=BLOCK):
    """Full N x N 0/1 mask of one head from its index list: M[r,c]=1 iff blk(c) listed for blk(r), c valid."""
    M = np.zeros((seq_len, seq_len), dtype=np.float64)
    nb = seq_len // block
    for i in range(nb):
        for j in idx[i, : cnt[i]]:
            M[i * block : (i + 1) * block, j * block : min((j + 1) * block, seq_valid)] = 1.0
    return M


def block_sparse_attn_head(Q, K, V, idx, cnt, seq_valid, scale=None, qblocks=None, block=BLOCK, block_valid=None):
    """Block-masked attention for one head.  Q,K,V: [N, d]; idx [nb,kmax], cnt [nb].

    For each query block i the keys with log M = 0 are exactly the valid tokens of the listed
    blocks; the softmax is taken over those keys (the others contribute exp(-inf) = 0).
    Returns O [N, d] fp64 and lse [N] fp64; rows of query blocks not in `qblocks` (default: all)
    are left at 0 / -inf, as are padded rows and rows of blocks with an empty list.
    block_valid: per-block valid counts (see block_scores); default: the first seq_valid tokens are valid."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    N, d = Q.shape
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    O = np.zeros((N, d))
    lse = np.full((N,), -np.inf)
    nb = N // block
    nv = _valid_counts(nb, seq_valid, block, block_valid)
    for i in range(nb) if qblocks is None else qblocks:
        r0, r1 = i * block, i * block + nv[i]
        if r1 <= r0 or cnt[i] == 0:
            continue
        cols = np.concatenate([np.arange(j * block, j * block + nv[j]) for j in idx[i, : cnt[i]]])
        if cols.size == 0:
            continue
        P, l = _softmax_rows((Q[r0:r1] @ K[cols].T) * scale)
        O[r0:r1] = P @ V[cols]
        lse[r0:r1] = l
    return O, lse


def block_sparse_attn(Q, K, V, idx, cnt, seq_valid, scale=None, block=BLOCK, block_valid=None):
    """All heads.  Q,K,V: [B,Hh,N,d]; idx [B,Hh,nb,kmax]; cnt [B,Hh,nb] -> O [B,Hh,N,d], lse [B,Hh,N] (fp64)."""
    B, Hh, N, d = Q.shape
    O = np.zeros((B, Hh, N, d))
    lse = np.full((B, Hh, N), -np.inf)
    for b in range(B):
        for h in range(Hh):
            O[b, h], lse[b, h] = block_sparse_attn_head(
                Q[b, h], K[b, h], V[b, h], idx[b, h], cnt[b, h], seq_valid, scale, None, block, block_valid
            )
    return O, lse


# --------------------------------------------------------------------------- #
# either side of the path: raster <-> cube-major token order (Figure 2, right)
# --------------------------------------------------------------------------- #
def cube_token_order(grid, cube):
    """order[p] = raster index t*H*W + h*W + w of the token at cube-major position p.

    grid = (T, H, W), cube = (ct, ch, cw).  Built by walking the cubes one by one: first every
    cube that fits wholly inside the grid, then the ones the boundary cuts, both in raster order
    of the cube coordinates; a cube's tokens in raster order of their local coordinates."""
    T, H, W = grid
    ct, ch, cw = cube
    cubes = [(a, b, c) for a in range(0, T, ct) for b in range(0, H, ch) for c in range(0, W, cw)]
    whole = [q for q in cubes if q[0] + ct <= T and q[1] + ch <= H and q[2] + cw <= W]
    cut = [q for q in cubes if q not in set(whole)]
    order = []
    for (a, b, c) in whole + cut:
        for t in range(a, min(a + ct, T)):
            for h in range(b, min(b + ch, H)):
                for w in range(c, min(c + cw, W)):
                    order.append((t * H + h) * W + w)
    return np.asarray(order, dtype=np.int64)


def cube_token_order_padded(grid, cube):
    """One cube per block, EVERY cube (Figure 2, right: Q, K and V are split into local 3-D cubes): the cubes
    in raster order of their cube coordinates, each given a block of ct*ch*cw positions; a cube the grid
    boundary cuts fills the first positions of its block with its tokens (raster order of the local coordinates
    inside the clipped cube) and leaves the rest as padding.
    Returns order [n_cubes * ct*ch*cw] (raster index, or -1 at a padding position) and valid [n_cubes]."""
    T, H, W = grid
    ct, ch, cw = cube
    size = ct * ch * cw
    order, valid = [], []
    for a in range(0, T, ct):
        for b in range(0, H, ch):
            for c in range(0, W, cw):
                toks = [(t * H + h) * W + w for t in range(a, min(a + ct, T)) for h in range(b, min(b + ch, H))
                        for w in range(c, min(c + cw, W))]
                valid.append(len(toks))
                order.extend(toks + [-1] * (size - len(toks)))
    return np.asarray(order, dtype=np.int64), np.asarray(valid, dtype=np.int64)


def order_gather(X, order):
    """X [..., tokens, d] -> [..., len(order), d]: row p is X[order[p]], or zero where order[p] < 0."""
    X = np.asarray(X)
    order = np.asarray(order)
    out = np.zeros(X.shape[:-2] + (len(order), X.shape[-1]), dtype=X.dtype)
    keep = order >= 0
    out[..., keep, :] = X[..., order[keep], :]
    return out


def order_scatter(Y, order, tokens):
    """The inverse of order_gather: out[order[p]] = Y[p] for the positions that hold a token."""
    Y = np.asarray(Y)
    order = np.asarray(order)
    keep = order >= 0
    out = np.zeros(Y.shape[:-2] + (tokens, Y.shape[-1]), dtype=Y.dtype)
    out[..., order[keep], :] = Y[..., keep, :]
    return out


def cube_gather(X, grid, cube, seq_len):
    """Raster-ordered X [..., T*H*W, d] -> cube-major [..., seq_len, d]; rows past T*H*W are zero."""
    X = np.asarray(X)
    order = cube_token_order(grid, cube)
    out = np.zeros(X.shape[:-2] + (seq_len, X.shape[-1]), dtype=X.dtype)
    out[..., : len(order), :] = X[..., order, :]
    return out


def cube_scatter(Y, grid, cube):
    """Cube-major Y [..., seq_len, d] -> raster order [..., T*H*W, d] (the padding rows are dropped)."""
    Y = np.asarray(Y)
    order = cube_token_order(grid, cube)
    out = np.empty(Y.shape[:-2] + (len(order), Y.shape[-1]), dtype=Y.dtype)
    out[..., order, :] = Y[..., : len(order), :]
    return out


# --------------------------------------------------------------------------- #
# cube-level branch and output fusion (Figure 2, right; Section 2.2's coarse level)
# --------------------------------------------------------------------------- #
def coarse_attn(S, V, seq_valid, block=BLOCK, block_valid=None):
    """C[b,h,i,:] = sum_j softmax_j(S[b,h,i,:])_j * mean(V_j) over the cubes holding a valid token.

    S: fp32 scores [B,Hh,nb,nb] (already scaled); V: [B,Hh,N,d].  Returns fp64 [B,Hh,nb,d];
    rows of cubes without a valid token are 0.  block_valid: per-block valid counts (see block_scores)."""
    S = _f64(S)
    nb = S.shape[-1]
    live = np.nonzero(_valid_counts(nb, seq_valid, block, block_valid) > 0)[0]
    Vm = block_means(V, seq_valid, block, block_valid)[..., live, :]
    L = S[..., live, :][..., live]
    P = np.exp(L - L.max(axis=-1, keepdims=True))
    P = P / P.sum(axis=-1, keepdims=True)
    C = np.zeros(S.shape[:-1] + (Vm.shape[-1],))
    C[..., live, :] = P @ Vm
    assert C.shape[-2] == nb
    return C


def fuse_outputs(fine, coarse, seq_valid, gate_fine=None, gate_coarse=None, block=BLOCK):
    """out[r] = gate_fine[r] * fine[r] + gate_coarse[r] * coarse[cube(r)] for r < seq_valid, else 0.

    fine, gates: [B,Hh,N,d]; coarse: [B,Hh,nb,d].  A missing gate is 1."""
    fine, coarse = _f64(fine), _f64(coarse)
    N = fine.shape[-2]
    spread = np.repeat(coarse, block, axis=-2)  # every token of cube i receives row i
    gf = 1.0 if gate_fine is None else _f64(gate_fine)
    gc = 1.0 if gate_coarse is None else _f64(gate_coarse)
    out = gf * fine + gc * spread
    out[..., seq_valid:, :] = 0.0
    assert out.shape[-2] == N
    return out


# --------------------------------------------------------------------------- #
# entropy-aware allocation of sparsity (Section 3.4)
# --------------------------------------------------------------------------- #
def attention_entropy(S, seq_valid, block=BLOCK):
    """Normalised entropy of the key marginal of the cube-level attention weights, one value per batch element.

    S: fp32 scores [B,Hh,nb,nb].  A = row softmax over the valid cubes; marginal a(j) = mean over heads
    and valid query cubes of A[h,i,j]; h = -sum_j a(j) log a(j) / log(n) with n the number of valid cubes."""
    S = _f64(S)
    n = (seq_valid + block - 1) // block
    L = S[..., :n, :n]
    A = np.exp(L - L.max(axis=-1, keepdims=True))
    A = A / A.sum(axis=-1, keepdims=True)
    a = A.mean(axis=(1, 2))  # [B, n]
    if n == 1:
        return np.zeros(S.shape[0])
    with np.errstate(divide="ignore", invalid="ignore"):
        terms = np.where(a > 0, a * np.log(a), 0.0)
    return -terms.sum(axis=-1) / math.log(n)


def entropy_allocate(h, rho_bar, gamma, rho_min, rho_max):
    """Per-layer sparsity from per-layer entropies h[l]: w = (1 - h)^gamma, rho[l] = clip(rho_bar * w[l] / mean(w))."""
    h = _f64(h)
    w = (1.0 - h) ** gamma
    if w.mean() == 0.0:
        # every layer at entropy 1: the ratio w / mean(w) is 0/0 and no layer is told apart from
        # another, so the base sparsity stands (Section 3.4 redistributes a budget, it does not create one)
        return np.clip(np.full(h.shape, float(rho_bar)), rho_min, rho_max)
    return np.clip(rho_bar * w / w.mean(), rho_min, rho_max)


# --------------------------------------------------------------------------- #
# token merging (Section 3.3)
# --------------------------------------------------------------------------- #
def merge_partition(grid, mblock):
    """dst[i] = raster index of the destination token of token i's merge block (dst[i] == i for destinations)."""
    T, H, W = grid
    st, sh, sw = mblock
    dst = np.empty(T * H * W, dtype=np.int64)
    for t in range(T):
        for h in range(H):
            for w in range(W):
                dst[(t * H + h) * W + w] = ((t - t % st) * H + (h - h % sh)) * W + (w - w % sw)
    return dst


def merge_similarity(K, grid, mblock):
    """u[b, i]: cosine similarity between the head-averaged key descriptors of source i and of its
    destination; -inf at the destinations themselves.  K: [B, Hh, N, d] in raster order."""
    m = _f64(K).mean(axis=1)  # head-averaged descriptors [B, N, d]
    dst = merge_partition(grid, mblock)
    norm = np.sqrt((m * m).sum(axis=-1))
    dot = (m * m[:, dst, :]).sum(axis=-1)
    den = norm * norm[:, dst]
    u = np.where(den > 0, dot / np.where(den > 0, den, 1.0), 0.0)
    u[:, dst == np.arange(len(dst))] = -np.inf
    return u


def merge_plan(u, grid, mblock, r):
    """From the similarities u [B, N] (fp32 values as handed over): which sources merge and where every
    token's features end up.  Returns row_of [B, N] (row of the merged sequence that token k reads back
    from: its own row, or its destination's if it was merged) and src_of [B, N - r] (raster index of
    the token that owns each merged row)."""
    u = np.asarray(u, dtype=np.float32)
    B, N = u.shape
    dst = merge_partition(grid, mblock)
    is_dst = dst == np.arange(N)
    sources = np.nonzero(~is_dst)[0]
    assert 0 <= r <= len(sources)
    row_of = np.empty((B, N), dtype=np.int32)
    src_of = np.empty((B, N - r), dtype=np.int32)
    for b in range(B):
        # u descending, then index ascending, on canonical values: -0 equals +0 (they compare equal as
        # floats) and NaN ranks after every number, as in the top-k selection
        order = sorted(sources.tolist(), key=lambda i: (bool(np.isnan(u[b, i])), 0.0 if np.isnan(u[b, i]) else -float(u[b, i]), i))
        merged = set(order[:r])
        unmerged = [i for i in sources.tolist() if i not in merged]
        seq = unmerged + np.nonzero(is_dst)[0].tolist()
        src_of[b] = seq
        pos = {tok: p for p, tok in enumerate(seq)}
        for k in range(N):
            row_of[b, k] = pos[int(dst[k])] if k in merged else pos[k]
    return row_of, src_of


def merge_apply(X, row_of, src_of, seq_len):
    """Merged features: row p is the mean of the features of every token that reads back from row p
    (a destination with its merged sources; an unmerged source alone).  X: [B, Hh, N, d] ->
    [B, Hh, seq_len, d] (fp64), rows past N - r are zero."""
    X = _f64(X)
    B, Hh, N, d = X.shape
    out = np.zeros((B, Hh, seq_len, d))
    for b in range(B):
        count = np.zeros(src_of.shape[1])
        acc = np.zeros((Hh, src_of.shape[1], d))
        for k in range(N):
            acc[:, row_of[b, k], :] += X[b, :, k, :]
            count[row_of[b, k]] += 1
        out[b, :, : src_of.shape[1], :] = acc / count[None, :, None]
    return out


def unmerge_apply(Y, row_of):
    """Token k takes row row_of[k] of the merged sequence.  Y: [B, Hh, seq_len, d] -> [B, Hh, N, d]."""
    Y = np.asarray(Y)
    return np.stack([Y[b][:, row_of[b], :] for b in range(Y.shape[0])])
