/*
 * usv.h - C ABI of the MI355X (gfx950) dynamic block-sparse video attention library.
 *
 * The library implements the attention hot path of a sparsified video diffusion
 * transformer in three calls:
 *
 *   usv_block_scores      coarse stage: one score per (query cube, key cube) pair
 *   usv_select_topk       per query cube, the k best key cubes -> compact index list
 *   usv_block_sparse_attn softmax attention over only the listed key/value cubes
 *
 * Tokens are the flattened 3-D video latent, ordered cube-major: the 64 tokens
 * of one 4x4x4 spatio-temporal cube are consecutive, so "block i" is tokens
 * [64 i, 64 i + 64).  usv_cube_gather / usv_cube_scatter convert from and to the
 * raster order a model holds its tokens in.
 *
 * Common conventions
 *   - Every pointer except the usv_shape is a DEVICE pointer to caller-owned
 *     memory (the library never allocates, frees or keeps a pointer), contiguous
 *     in the stated layout with the last index fastest, 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it; they never synchronise the host.
 *   - Arguments are validated on the host before anything is launched; a call
 *     that returns an error has launched nothing.  Errors are status codes, never
 *     aborts.  usv_last_error() gives a message for the calling thread's last error.
 *   - Device contents are not validated (index lists, budgets): see each call.
 *   - Padded tokens (seq_valid <= token < seq_len) may hold any FINITE values.
 */
#ifndef USV_H
#define USV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  USV_OK = 0,
  USV_ERR_INVALID_ARG = 1, /* null/misaligned pointer, inconsistent sizes */
  USV_ERR_UNSUPPORTED = 2, /* block != 64, head_dim not in {64,128}, too many blocks */
  USV_ERR_WORKSPACE = 3,   /* workspace missing or smaller than usv_workspace_bytes */
  USV_ERR_HIP = 4          /* the HIP runtime refused a launch */
} usv_status;

typedef enum { USV_F32 = 0, USV_BF16 = 1 } usv_dtype;

/* Problem shape shared by the three stages (host struct). */
typedef struct {
  int32_t batch;     /* B  >= 1 */
  int32_t heads;     /* Hh >= 1 (attention heads) */
  int32_t seq_len;   /* N: padded token count, a multiple of `block` */
  int32_t seq_valid; /* Nv: real tokens, N - block < Nv <= N is typical; 1 <= Nv <= N */
  int32_t head_dim;  /* d: 64 or 128 */
  int32_t block;     /* tokens per cube: 64 */
  int32_t dtype;     /* usv_dtype of Q, K, V */
} usv_shape;

#define USV_MAX_BLOCKS 4096 /* largest supported N / block */

/* Bytes of device scratch usv_block_scores needs for `shape` (pooled fp32 means
 * of Q and K: 2 * B * Hh * nb * d * 4).  Returns 0 for an invalid shape. */
size_t usv_workspace_bytes(const usv_shape* shape);

/*
 * Stage 1 - pooled block scores (the coarse stage of the coarse-to-fine sparse
 * attention the paper builds on, Section 2.2 / Section 3.2; Figure 2 "3D cubes").
 *
 *   Qm[b,h,i,:] = mean over valid tokens r of block i of Q[b,h,r,:]   (fp32)
 *   Km[b,h,j,:] likewise
 *   scores[b,h,i,j] = Qm[b,h,i,:] . Km[b,h,j,:] / sqrt(d)             (fp32)
 *
 * q, k   : [B, Hh, N, d] of shape->dtype (device, read only)
 * scores : [B, Hh, nb, nb] fp32 (device, written); rows and columns of blocks
 *          that hold no valid token are written as -inf
 * ws     : device scratch of at least usv_workspace_bytes(shape) bytes; its
 *          contents on return are unspecified
 */
usv_status usv_block_scores(const void* q, const void* k, const usv_shape* shape,
                            float* scores, void* ws, size_t ws_bytes, void* stream);

/*
 * usv_block_scores for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * same kernels, with the pooled means kept in a static device array of
 * USV_STATIC_SCRATCH_BYTES that is part of the library image instead of in a
 * caller workspace.  The call allocates and frees nothing; the caller still
 * passes q, k and scores.  Same results as usv_block_scores, bit for bit.
 *
 * Limit: usv_workspace_bytes(shape) <= USV_STATIC_SCRATCH_BYTES (64 MiB; the
 * 480p shape needs 6.3 MB, the 720p shape 48.4 MB), else USV_ERR_WORKSPACE and
 * nothing is launched.  Every GPU the library is used on holds its own copy of
 * the array until the process ends.  All calls on one GPU share that copy:
 * calls that can overlap on one GPU (different streams, different threads)
 * race on it and must be ordered by the caller.  The first call on a device
 * looks the array's address up (no allocation); make that call outside graph
 * capture.
 */
#define USV_STATIC_SCRATCH_BYTES (64u << 20)
usv_status usv_block_scores_static(const void* q, const void* k, const usv_shape* shape,
                                   float* scores, void* stream);

/*
 * Stage 2 - per-query-block top-k key-block selection ("top-k cube selection",
 * Figure 2).  For every row (b, h, i) with i a block holding a valid token:
 *   candidates = key blocks j that hold a valid token
 *   keep       = min(budget, kmax, #candidates), budget = budgets[b,h,i] if
 *                budgets != NULL else k; a negative budget counts as 0
 *   order      = score descending, then block index ascending, on canonical
 *                values: -0 equals +0 and NaN ranks below -inf
 * The kept indices are written in ASCENDING block index to idx[b,h,i,0..keep),
 * the remaining slots up to kmax hold -1, and cnt[b,h,i] = keep.  Rows of blocks
 * without a valid token get cnt = 0.
 *
 * scores  : [B, Hh, nb, nb] fp32 (device, read only)
 * k       : uniform budget (1 <= k <= kmax) when budgets == NULL, else ignored
 * budgets : NULL or [B, Hh, nb] int32 (device, read only)
 * kmax    : row stride of idx, 1 <= kmax <= nb
 * idx     : [B, Hh, nb, kmax] int32 (device, written)
 * cnt     : [B, Hh, nb] int32 (device, written)
 * Only shape->batch/heads/seq_len/seq_valid/block are used.
 */
usv_status usv_select_topk(const float* scores, const usv_shape* shape, int32_t k,
                           const int32_t* budgets, int32_t kmax, int32_t* idx, int32_t* cnt,
                           void* stream);

/* usv_select_topk with options.  flags = 0 is usv_select_topk itself.
 * USV_TOPK_FORCE_LOCAL (Figure 2, right: the budget is split between attention inside
 * the local cube and sparse attention to far-away cubes): a row that keeps anything keeps
 * its OWN cube i, and fills the rest of its budget with the best other cubes in
 * the order above.  The paper gives no rule for the split; this reading spends
 * one block of the budget on the local cube. */
#define USV_TOPK_FORCE_LOCAL 1u
usv_status usv_select_topk_ex(const float* scores, const usv_shape* shape, int32_t k,
                              const int32_t* budgets, int32_t kmax, uint32_t flags, int32_t* idx,
                              int32_t* cnt, void* stream);

/*
 * Stage 3 - block-sparse attention: the masked-attention equation of Section 3.2,
 *   out = softmax(Q K^T * scale + log M) V,
 * with M[r, c] = 1 iff block(c) is listed for block(r) and c < seq_valid.
 * Only the listed K/V blocks are read (Section 2.2: attention is dense inside the
 * selected tiles and absent elsewhere).  With every block listed this is the dense-attention
 * equation of the same section.
 *
 * q, k, v : [B, Hh, N, d] of shape->dtype (device, read only)
 * idx     : [B, Hh, nb, kmax] int32; row (b,h,i) holds cnt[b,h,i] DISTINCT block
 *           ids in [0, ceil(Nv/64)) in its first slots, in any order (ascending
 *           reads K/V most cache-friendly).  Device contents are not validated:
 *           ids outside [0, nb) and counts outside [0, kmax] are clamped into
 *           range, so no memory outside the tensors is touched, but the rows of
 *           such a list hold unspecified values.
 * cnt     : [B, Hh, nb] int32, 0 <= cnt <= kmax
 * scale   : softmax scale; <= 0 selects 1/sqrt(d)
 * out_dtype : usv_dtype of `out`: shape->dtype, or USV_F32 for bf16 inputs (the
 *           fp32 accumulator is then stored unrounded; rounding the result to
 *           bf16 costs up to half a bf16 ulp, 2^-9 relative, on top of the
 *           kernel's own error)
 * out     : [B, Hh, N, d] of out_dtype (written).  Rows of padded tokens and of
 *           query blocks with cnt = 0 are written as 0.
 * lse     : NULL or [B, Hh, N] fp32 (written): natural-log sum of exp of the
 *           scaled logits over the row's allowed keys; -inf where out is 0.
 * bf16 inputs: QK^T and PV run on bf16 MFMA with fp32 accumulation and an fp32
 * online softmax; the probabilities are rounded to bf16 before PV and the row
 * sums are taken over the rounded values.
 * fp32 inputs: both products on the fp32 matrix cores (fp32 operands and
 * accumulation), fp32 softmax: within 1e-5 relative of an fp64 evaluation.
 */
usv_status usv_block_sparse_attn(const void* q, const void* k, const void* v,
                                 const usv_shape* shape, const int32_t* idx, const int32_t* cnt,
                                 int32_t kmax, float scale, int32_t out_dtype, void* out, float* lse,
                                 void* stream);

/*
 * Work order of the attention launch.  Stage 3 is the same whichever query
 * block a workgroup takes, so its launch may walk the query blocks of a head in
 * any order.  Walking them sorted by
 *     (list length descending, where the list lies ascending, block index)
 * keeps the workgroups that run together on lists of similar length and
 * similar placement: their ascending sweeps over the head's K/V then stay
 * together in the 4 MiB L2 of the XCD they share, and the last round of the
 * launch is made of the shortest lists.  "Where the list lies" = its entries at
 * 1/4, 1/2 and 3/4 of its length, each reduced to one of 64 equal buckets of
 * the block range, compared lexicographically.  Measured on MI355X: per-row
 * budgets uniform in 8..64 at the merged 480p shape 12 % faster than index
 * order; uniform budgets at the 720p shape (59 of 1182 blocks, where a head's
 * K and V are ten times the L2) 20 % faster; uniform budgets at the 480p shape
 * 1 % (there the sort costs what it gains).  It pays when the lists are ragged
 * or when a head's K and V are many times the L2.
 *
 *   usv_attn_work_order   work_order[b,h,s] = the query block that slot s of head
 *                         (b,h) takes; deterministic.  idx == NULL: by list
 *                         length (and block index) only.
 *   usv_block_sparse_attn_ordered   usv_block_sparse_attn with that table;
 *                         work_order == NULL is usv_block_sparse_attn.  The
 *                         output does not depend on the table as long as every
 *                         head's slice is a permutation of 0..nb-1 (entries are
 *                         clamped into range; a block named twice is computed
 *                         twice, a block never named is not written).  fp32
 *                         inputs ignore the table.
 * idx        : NULL or [B, Hh, nb, kmax] int32 (device, read only), ascending lists
 *              as written by stage 2 (other lists only make the order less useful)
 * cnt        : [B, Hh, nb] int32 (device, read only), as written by stage 2
 * work_order : [B, Hh, nb] int32 (device)
 */
usv_status usv_attn_work_order(const int32_t* idx, const int32_t* cnt, const usv_shape* shape,
                               int32_t kmax, int32_t* work_order, void* stream);
usv_status usv_block_sparse_attn_ordered(const void* q, const void* k, const void* v,
                                         const usv_shape* shape, const int32_t* idx,
                                         const int32_t* cnt, int32_t kmax,
                                         const int32_t* work_order, float scale, int32_t out_dtype,
                                         void* out, float* lse, void* stream);

/*
 * Cube-level branch and fusion (Figure 2, right: each branch's result is spread over
 * the whole token grid again and the branches are then combined into one output;
 * Section 2.2: the coarse level of the coarse-to-fine scheme).  The paper prints
 * no formula for either; the readings, following the coarse-to-fine sparse
 * attention it builds on:
 *   coarse[b,h,i,:] = sum_j softmax_j(scores[b,h,i,:])_j * mean(V cube j)
 *                     over the cubes j that hold a valid token (scores as written
 *                     by usv_block_scores: they already carry 1/sqrt(d));
 *   out[b,h,r,:]    = gate_fine[b,h,r,:] * fine[b,h,r,:]
 *                   + gate_coarse[b,h,r,:] * coarse[b,h,r/64,:]   (elementwise),
 * i.e. every token of cube i receives row i of the cube-level output, and the
 * model supplies per-token, per-channel gates (NULL gate = 1).
 */

/* Bytes of device scratch usv_coarse_attn needs (pooled fp32 means of V:
 * B * Hh * nb * d * 4).  Returns 0 for an invalid shape. */
size_t usv_coarse_workspace_bytes(const usv_shape* shape);

/* scores : [B, Hh, nb, nb] fp32 (device, read only), from usv_block_scores
 * v      : [B, Hh, N, d] of shape->dtype (device, read only)
 * coarse : [B, Hh, nb, d] fp32 (device, written); rows of cubes without a valid
 *          token are written as 0
 * ws     : device scratch >= usv_coarse_workspace_bytes(shape); contents unspecified on return */
usv_status usv_coarse_attn(const float* scores, const void* v, const usv_shape* shape, float* coarse,
                           void* ws, size_t ws_bytes, void* stream);

/* fine        : [B, Hh, N, d] of fine_dtype (the output of usv_block_sparse_attn)
 * coarse      : [B, Hh, nb, d] fp32 (from usv_coarse_attn)
 * gate_fine, gate_coarse : NULL or [B, Hh, N, d] of shape->dtype (device, read only)
 * out         : [B, Hh, N, d] of out_dtype (written; bf16 results are rounded to
 *               nearest even from the fp32 sum).  Rows of padded tokens are 0.
 *               out may be the same buffer as fine when out_dtype == fine_dtype;
 *               any other overlap is undefined. */
usv_status usv_fuse_outputs(const void* fine, int32_t fine_dtype, const float* coarse,
                            const void* gate_fine, const void* gate_coarse, const usv_shape* shape,
                            int32_t out_dtype, void* out, void* stream);

/*
 * Entropy-aware allocation of sparsity (Section 3.4).  The paper averages the
 * attention weights over heads and queries into a marginal over keys, takes its
 * entropy normalised by log N, turns it into a weight (1 - h)^gamma and spreads
 * a base sparsity over the layers in proportion to the weights, clipped.
 * The full N x N weights are never formed by a sparse kernel and the paper does
 * not say where it takes them from; here they are the cube-level weights
 *   A[b,h,i,:] = softmax_j(scores[b,h,i,:]) over the cubes j with a valid token,
 *   a[b,j]     = mean over h and valid i of A[b,h,i,j],
 *   entropy[b] = - sum_j a[b,j] log a[b,j] / log n,   n = number of valid cubes
 * (0 log 0 = 0; n = 1 gives 0).  With one token per cube this is the paper's
 * definition exactly.
 */

/* Bytes of device scratch usv_attn_entropy needs (per-tile column sums:
 * B * Hh * ceil(nb_valid / 32) * nb * 4).  Returns 0 for an invalid shape. */
size_t usv_entropy_workspace_bytes(const usv_shape* shape);

/* scores  : [B, Hh, nb, nb] fp32 (device, read only), from usv_block_scores
 * entropy : [B] fp32 (device, written), each in [0, 1]
 * ws      : device scratch >= usv_entropy_workspace_bytes(shape)
 * Only shape->batch/heads/seq_len/seq_valid/block are used.  The summation order
 * is fixed: the result is bit-reproducible. */
usv_status usv_attn_entropy(const float* scores, const usv_shape* shape, float* entropy, void* ws,
                            size_t ws_bytes, void* stream);

/* HOST helper, launches nothing.  entropy[l], l < layers: the entropies of the
 * layers of one diffusion step (host array, each in [0, 1]).
 *   w[l]   = (1 - entropy[l])^gamma,            gamma >= 1
 *   rho[l] = clip(rho_min, rho_max, rho_bar * w[l] / mean_l(w))
 * Without clipping the mean of rho over the layers is rho_bar.  If every weight
 * is 0, rho[l] = clip(rho_bar).  A sparsity rho turns into a per-row budget as
 * k = max(1, floor((1 - rho) * nb)) in the caller. */
usv_status usv_entropy_allocate(const float* entropy, int32_t layers, float rho_bar, float gamma,
                                float rho_min, float rho_max, float* rho);

/*
 * Either side of the three stages: the token order (Figure 2, right: queries, keys
 * and values are split into small 3-D cubes, and the outputs are spread over the whole
 * token grid again).  A model holds tokens in raster order of the latent
 * grid, index (t*H + h)*W + w; the stages above want cube-major order.
 *
 * Cube-major order of a T x H x W grid tiled by ct x ch x cw cubes (ct*ch*cw = 64):
 *   1. the cubes that lie wholly inside the grid, in raster order of their cube
 *      coordinates (t/ct, h/ch, w/cw): whole cube number n is block n, tokens
 *      [64 n, 64 n + 64);
 *   2. then the cubes the grid boundary cuts, in the same raster order, packed
 *      without gaps, so that the only padding is the tail [T*H*W, seq_len);
 *   3. inside a cube, tokens in raster order of their local coordinates.
 * The paper does not say how a grid that the cube does not divide is tiled; this
 * reading keeps every whole cube one aligned block and leaves the padding where
 * seq_valid expects it.
 */

/* Token grid and cube (host struct). */
typedef struct {
  int32_t T, H, W;    /* latent grid, T*H*W == shape->seq_valid (merge calls: see there) */
  int32_t ct, ch, cw; /* cube, ct*ch*cw == shape->block (in the merge calls: the merge block, any size) */
} usv_grid;

/* Element strides of a raster-ordered tensor whose channel index is contiguous
 * (host struct): element (b, head, token, c) is at b*batch + head*head + token*token + c.
 * Each stride times the element size must be a multiple of 16 bytes and rows must not
 * overlap.  [B, Hh, Nv, d] is {Hh*Nv*d, Nv*d, d}; a projection output [B, Nv, Hh*d]
 * is {Nv*Hh*d, d, Hh*d}. */
typedef struct {
  int64_t batch, head, token;
} usv_strides;

/* HOST helper: order[p] = raster index of the token at cube-major position p, for
 * p in [0, T*H*W).  `order` is a host array of T*H*W int32.  Launches nothing. */
usv_status usv_cube_token_order(const usv_grid* grid, int32_t* order);

/*
 * Raster -> cube-major (with padding).  cube[b,h,p,:] = raster[b,h,order[p],:] for
 * p < T*H*W; rows T*H*W <= p < seq_len are written as zero.
 * raster  : device, read only, laid out by `strides` (NULL = contiguous [B,Hh,Nv,d])
 * shape   : seq_valid = T*H*W; dtype = element type of THIS tensor (an fp32
 *           attention output is moved with dtype = USV_F32)
 * cube    : [B, Hh, seq_len, d] contiguous (device, written); must not overlap raster
 */
usv_status usv_cube_gather(const void* raster, const usv_strides* strides, const usv_shape* shape,
                           const usv_grid* grid, void* cube, void* stream);

/* Cube-major -> raster, the inverse: raster[b,h,order[p],:] = cube[b,h,p,:] for
 * p < T*H*W; the padding rows of `cube` are not read.  Arguments as above, with
 * `raster` written and `cube` read only. */
usv_status usv_cube_scatter(const void* cube, const usv_shape* shape, const usv_grid* grid,
                            void* raster, const usv_strides* strides, void* stream);

/*
 * The three stages on RASTER-order tensors, with no reordered copy of anything:
 * the kernels look every token row up through the order table while they load
 * and store (the tile requests of the attention kernel carry per-lane global
 * addresses anyway).  Same results as usv_cube_gather -> stage -> usv_cube_scatter.
 *   usv_cube_order                the table on the device: order[p] = raster index
 *                                 of cube-major position p, p < seq_valid; the
 *                                 padding positions hold 0
 *   usv_block_scores_raster       usv_block_scores on raster Q, K
 *   usv_select_topk               unchanged (it only sees the scores)
 *   usv_block_sparse_attn_raster  usv_block_sparse_attn on raster Q, K, V, writing
 *                                 out (and lse, [B, Hh, seq_valid]) in raster order
 */
typedef struct {
  const int32_t* order;    /* device, [seq_len] int32, from usv_cube_order (any permutation works); NOT validated:
                              every entry is used as a token index and must lie in [0, seq_valid) */
  usv_strides in_strides;  /* element strides of q, k, v; token == 0 means contiguous [B, Hh, Nv, d] */
  usv_strides out_strides; /* element strides of out; token == 0 means contiguous [B, Hh, Nv, d] */
  const int32_t* block_valid; /* NULL, or device [seq_len / 64] int32 from usv_cube_order_padded: see there */
  const int32_t* work_order;  /* NULL, or device [B, Hh, seq_len / 64] int32 from usv_attn_work_order: the attention
                                 launch walks each head's query blocks in that order (same output) */
} usv_raster;

usv_status usv_cube_order(const usv_shape* shape, const usv_grid* grid, int32_t* order, void* stream);

/*
 * One cube per block, EVERY cube (Figure 2, right: Q, K and V are split into
 * local 3-D cubes): where usv_cube_order packs the cubes that the grid boundary
 * cuts, this table gives each of them a 64-position block of its own, in raster
 * order of the cube coordinates, so that every block's pooled mean, score and
 * selection is a quantity of ONE cube.  Block b holds the block_valid[b] tokens
 * of cube b in its first positions (raster order of the local coordinates inside
 * the clipped cube); the rest of the block is padding, and order[] holds 0 there
 * (a readable row; block_valid says that it does not count).
 *   blocks   = usv_cube_count(grid) = ceil(T/ct) * ceil(H/ch) * ceil(W/cw)
 *   order    : device, [64 * blocks] int32 (written)
 *   block_valid : device, [blocks] int32 (written), every entry in 1..64
 * Use: the raster entry points with shape->seq_len = 64 * blocks,
 * shape->seq_valid = T*H*W (the raster tensors' token count) and
 * view->block_valid set; usv_select_topk on these scores takes seq_valid =
 * seq_len (every block is a candidate).  With view->block_valid the kernels
 * average over a block's first block_valid[i] rows, mask the other keys, and
 * neither compute nor store the other query rows.
 */
int32_t usv_cube_count(const usv_grid* grid); /* 0 for an invalid grid */
usv_status usv_cube_order_padded(const usv_grid* grid, int32_t* order, int32_t* block_valid,
                                 void* stream);

/* Arguments as usv_block_scores; q, k laid out by view->in_strides. */
usv_status usv_block_scores_raster(const void* q, const void* k, const usv_shape* shape,
                                   const usv_raster* view, float* scores, void* ws, size_t ws_bytes,
                                   void* stream);

/* Arguments as usv_block_sparse_attn; bf16 inputs only (USV_ERR_UNSUPPORTED
 * otherwise); seq_valid * token stride must stay below 2 GiB.  out has seq_valid
 * rows per head (no padding rows), laid out by view->out_strides. */
usv_status usv_block_sparse_attn_raster(const void* q, const void* k, const void* v,
                                        const usv_shape* shape, const usv_raster* view,
                                        const int32_t* idx, const int32_t* cnt, int32_t kmax,
                                        float scale, int32_t out_dtype, void* out, float* lse,
                                        void* stream);

/* The second branch on raster-order tensors.
 * usv_coarse_attn_raster: usv_coarse_attn with v laid out by view->in_strides (any
 *   dtype usv_coarse_attn takes); coarse is [B, Hh, nb, d] fp32 as there.
 * usv_block_sparse_attn_raster_fused: usv_block_sparse_attn_fused on raster tensors
 *   (bf16 only); gate_fine and gate_coarse, where given, are raster-order bf16
 *   tensors laid out like q (view->in_strides).  Same results as gathering every
 *   tensor, calling the cube-major entry point and scattering the output. */
usv_status usv_coarse_attn_raster(const float* scores, const void* v, const usv_shape* shape,
                                  const usv_raster* view, float* coarse, void* ws, size_t ws_bytes,
                                  void* stream);
usv_status usv_block_sparse_attn_raster_fused(const void* q, const void* k, const void* v,
                                              const usv_shape* shape, const usv_raster* view,
                                              const int32_t* idx, const int32_t* cnt, int32_t kmax,
                                              float scale, const float* coarse, const void* gate_fine,
                                              const void* gate_coarse, int32_t out_dtype, void* out,
                                              float* lse, void* stream);

/*
 * Token merging (Section 3.3, "Token merging for video").  Tokens are in RASTER
 * order of the T x H x W grid.  The grid is tiled from the origin by merge blocks
 * of s_t x s_h x s_w tokens (usv_grid.ct/ch/cw; cut at the boundary).  The first
 * token of a block (local 0,0,0) is its destination, the others are sources.
 *   descriptor  m_i = mean over heads of K[b,h,i,:]                       (fp32)
 *   similarity  u_i = cos(m_i, m_dst(i)) for a source i, -inf for a destination
 *               (the paper restricts sources and destinations to local 3-D blocks:
 *               a source's only candidate is the destination of its own block;
 *               a zero descriptor gives 0)
 *   selection   the r sources first in the order (u descending, index ascending)
 *               are merged into their destinations; r <= number of sources
 *   merge       destination row = mean of its own and its merged sources' rows;
 *               unmerged sources keep theirs
 *   sequence    [unmerged sources, ascending index] then [destinations, ascending
 *               index]: N - r rows
 *   unmerge     token k reads its own row, a merged source its destination's row
 * In these calls `shape` describes the MERGED tensors: seq_valid = N - r rows are
 * real, seq_len (a multiple of 64) is the padded row count; r is therefore
 * T*H*W - seq_valid.  Raster tensors are contiguous [B, Hh, T*H*W, d].  After
 * merging, the three stages run on the merged tensors with the same shape.
 */

/* Bytes of device scratch usv_merge_similarity needs (descriptors and their
 * squared norms: B * T*H*W * (d + 1) * 4).  Returns 0 for invalid arguments. */
size_t usv_merge_workspace_bytes(const usv_shape* shape, const usv_grid* grid);

/* k   : [B, Hh, T*H*W, d] of shape->dtype, raster order (device, read only)
 * u   : [B, T*H*W] fp32 (device, written)
 * blk : [T*H*W] int32 (device, written): the partition, a function of the grid
 *       only: blk[i] & 0x7fffffff = rank of token i's merge block among the
 *       destinations in ascending raster order; bit 31 is set iff token i is the
 *       destination of its block */
usv_status usv_merge_similarity(const void* k, const usv_shape* shape, const usv_grid* grid, float* u,
                                int32_t* blk, void* ws, size_t ws_bytes, void* stream);

/* u      : [B, T*H*W] fp32 (device, read only); compared on canonical values
 *          (-0 equals +0, NaN ranks lowest); values at destinations are ignored;
 *          the result is a pure function of u and the grid
 * blk    : [T*H*W] int32 as written by usv_merge_similarity (device, read only;
 *          not validated)
 * row_of : [B, T*H*W] int32 (device, written): the merged row token k reads back
 * src_of : [B, N - r] int32 (device, written): the raster index of the token that
 *          owns each merged row
 * ws     : NULL, or device scratch of at least usv_merge_plan_workspace_bytes
 *          bytes (contents on return unspecified).  Without it one workgroup per
 *          batch element does the whole selection (fine for a few thousand
 *          tokens); with it the selection is a radix select spread over the chip
 *          (five short launches), which is what video-sized grids want.  The
 *          result is the same, bit for bit. */
size_t usv_merge_plan_workspace_bytes(const usv_shape* shape, const usv_grid* grid);
usv_status usv_merge_plan(const float* u, const int32_t* blk, const usv_shape* shape,
                          const usv_grid* grid, int32_t* row_of, int32_t* src_of,
                          void* ws, size_t ws_bytes, void* stream);

/* x      : [B, Hh, T*H*W, d] of shape->dtype, raster order (device, read only)
 * row_of, src_of : as written by usv_merge_plan for the same shape and grid (device,
 *       read only; not validated).  The layout of the merged sequence is relied on:
 *       the destinations own its last rows in ascending raster order, and row p of
 *       the others is a copy of token src_of[p].
 * out    : [B, Hh, seq_len, d] of shape->dtype (device, written); means are taken in
 *       fp32 and rounded once; rows seq_valid <= p < seq_len are written as zero */
usv_status usv_merge_apply(const void* x, const usv_shape* shape, const usv_grid* grid,
                           const int32_t* row_of, const int32_t* src_of, void* out, void* stream);

/* y   : [B, Hh, seq_len, d] of shape->dtype (device, read only)
 * out : [B, Hh, T*H*W, d] of shape->dtype (device, written): out[k] = y[row_of[k]]
 *       (shape->dtype is the element type of THIS tensor, e.g. USV_F32 for an fp32
 *       attention output) */
usv_status usv_unmerge_apply(const void* y, const usv_shape* shape, const usv_grid* grid,
                             const int32_t* row_of, void* out, void* stream);

/*
 * usv_block_sparse_attn with the second branch folded into its store, so that the
 * attention output never makes a round trip through memory:
 *   out = gate_fine * attention + gate_coarse * coarse[b,h,token/64,:]
 * exactly as usv_block_sparse_attn followed by usv_fuse_outputs with an fp32
 * intermediate.  coarse = NULL (then both gates must be NULL) is plain
 * usv_block_sparse_attn.  coarse: [B, Hh, nb, d] fp32; gates: NULL (= 1) or
 * [B, Hh, N, d] of shape->dtype.  lse, if requested, is the attention's.
 */
usv_status usv_block_sparse_attn_fused(const void* q, const void* k, const void* v,
                                       const usv_shape* shape, const int32_t* idx, const int32_t* cnt,
                                       int32_t kmax, float scale, const float* coarse,
                                       const void* gate_fine, const void* gate_coarse,
                                       int32_t out_dtype, void* out, float* lse, void* stream);

/* Static string for a status code. */
const char* usv_status_string(int32_t status);

/* Message describing the calling thread's most recent error ("" if none). */
const char* usv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* USV_H */
