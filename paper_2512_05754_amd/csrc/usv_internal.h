// Internal declarations shared by the HIP sources of libusv (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "usv.h"

namespace usv {

constexpr int kBlock = 64;        // tokens per cube
constexpr int kNumXcd = 8;        // MI355X: 8 accelerator dies, each with its own L2
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct Dims {
  int B, Hh, N, Nv, d, nb, nb_valid;
  bool bf16;
  long long bh() const { return (long long)B * Hh; }
};

// Token grid T x H x W tiled by ct x ch x cw cubes; Tf, Hf, Wf = whole cubes along each axis.
struct CubeGrid {
  int T, H, W, ct, ch, cw, Tf, Hf, Wf;
};
// Cube-major position of raster token (t, h, w): the one definition the kernel and the host helper share.
__host__ __device__ long long cube_position(const CubeGrid& g, int t, int h, int w);

// Token grid T x H x W tiled by st x sh x sw merge blocks (cut at the boundary); nT, nH, nW = blocks along each axis.
struct MergeGrid {
  int T, H, W, st, sh, sw, nT, nH, nW;
};

// Workgroups are dealt round-robin to the 8 XCDs.  Map the hardware block id to a logical
// work id so that each XCD walks one contiguous range of work items (consecutive heads and
// query blocks share K/V in that XCD's L2).  `per_xcd` = ceil(total / 8); ids >= total idle.
__device__ __forceinline__ int xcd_contiguous_id(int bid, int per_xcd) {
  return (bid % kNumXcd) * per_xcd + bid / kNumXcd;
}

// launchers (each returns the hipError_t of its launches)

hipError_t launch_select_topk(const float* scores, const Dims& s, int k, const int32_t* budgets, int kmax,
                              bool force_local, int32_t* idx, int32_t* cnt, hipStream_t st);
struct RasterArgs;
hipError_t launch_pool_means(const void* x, const Dims& s, float* means, hipStream_t st,
                             const RasterArgs* ras = nullptr);  // ras == nullptr: cube-major x
hipError_t launch_coarse_attn(const float* scores, const float* vmean, const Dims& s, float* coarse, hipStream_t st);
hipError_t launch_attn_entropy(const float* scores, const Dims& s, float* entropy, float* ws, hipStream_t st);
hipError_t launch_fuse_outputs(const void* fine, bool fine_f32, const float* coarse, const void* gate_fine,
                               const void* gate_coarse, bool gates_f32, void* out, bool out_f32, const Dims& s,
                               hipStream_t st);
hipError_t launch_attn_f32(const float* q, const float* k, const float* v, const Dims& s, const int32_t* idx,
                           const int32_t* cnt, int kmax, float scale, float* out, float* lse, hipStream_t st);
// Optional second branch folded into the attention kernel's store (all NULL: plain attention):
// out = gate_fine * attention + gate_coarse * coarse[cube]; a NULL gate is 1.  Gates are bf16 [B,Hh,N,d].
struct FuseArgs {
  const float* coarse;
  const uint16_t* gate_fine;
  const uint16_t* gate_coarse;
};
// Raster-order tensors for the attention and pooling kernels: order[p] = raster index of cube-major position p
// (padding positions hold any valid index); strides in BYTES; the output has its own strides.
// block_valid == nullptr: the first Nv positions hold tokens.  Otherwise block i holds block_valid[i] tokens in
// its first positions (one cube per block, cut cubes padded) and the rest of the block is padding.
struct RasterArgs {
  const int32_t* order;
  long long tok, head, batch;
  long long o_tok, o_head, o_batch;
  int Hh;
  const int32_t* block_valid;
};
// ras == nullptr: cube-major Q, K
hipError_t launch_block_scores(const void* q, const void* k, const Dims& s, float* scores, float* ws,
                               hipStream_t st, const RasterArgs* ras = nullptr);
hipError_t launch_attn_bf16_raster(const void* q, const void* k, const void* v, const Dims& s, const RasterArgs& ras,
                                   const int32_t* idx, const int32_t* cnt, int kmax, float scale, void* out,
                                   bool out_f32, float* lse, const FuseArgs& fuse, hipStream_t st,
                                   const int32_t* work_order = nullptr);
// work_order == nullptr: workgroup slot s of a head takes query block s; otherwise block work_order[head * nb + s]
hipError_t launch_attn_bf16(const void* q, const void* k, const void* v, const Dims& s, const int32_t* idx,
                            const int32_t* cnt, int kmax, float scale, void* out, bool out_f32, float* lse,
                            const FuseArgs& fuse, hipStream_t st, const int32_t* work_order = nullptr);
hipError_t launch_attn_work_order(const int32_t* idx, const int32_t* cnt, const Dims& s, int kmax, int32_t* work_order,
                                  hipStream_t st);  // idx == nullptr: by list length only

// gather: raster -> cube-major (+ zeroed padding); else cube-major -> raster.  Strides of the raster tensor in BYTES.
hipError_t launch_cube_order(int32_t* order, const CubeGrid& g, int N, int Nv, hipStream_t stream);
hipError_t launch_cube_order_padded(int32_t* order, int32_t* block_valid, const CubeGrid& g, hipStream_t stream);
hipError_t launch_cube_move(bool gather, const void* src, void* dst, const CubeGrid& g, const Dims& s, long long sb,
                            long long sh, long long st, hipStream_t stream);

// Token merging.  `s` describes the MERGED tensors (s.N padded rows, s.Nv = N - r valid rows); N = raster tokens.
hipError_t launch_merge_similarity(const void* k, const Dims& s, const MergeGrid& g, int N, float* u, int32_t* blk,
                                   float* ws, hipStream_t st);
size_t merge_plan_workspace_bytes(int B, int N);
hipError_t launch_merge_select(const float* u, const int32_t* blk, const MergeGrid& g, int B, int N, int r, int32_t* row_of,
                               int32_t* src_of, void* ws, hipStream_t st);
hipError_t launch_merge_rows(const void* x, const Dims& s, const MergeGrid& g, int N, const int32_t* row_of,
                             const int32_t* src_of, void* out, hipStream_t st);
hipError_t launch_unmerge_rows(const void* y, const Dims& s, int N, const int32_t* row_of, void* out, hipStream_t st);

}  // namespace usv
