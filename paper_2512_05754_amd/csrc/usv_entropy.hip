// Entropy of the key marginal of the cube-level attention weights (paper Section 3.4: the marginal
// of the attention weights over heads and queries, and its entropy normalised by log N).
//   A[h,i,:] = softmax_j(S[h,i,:]) over the cubes with a valid token (S = stage-1 scores)
//   a(j)     = mean over heads h and valid query cubes i of A[h,i,j]
//   h        = - sum_j a(j) log a(j) / log(n),  n = number of valid cubes
// Two kernels, both deterministic (fixed summation order, no atomics):
//   entropy_partials  one workgroup per 32 score rows of a head: row max and row sum, then the
//                     column sums of the 32 normalised rows -> partial[bh][tile][j]
//   entropy_finish    one workgroup per batch element: adds the partials of all heads and tiles,
//                     forms a(j) log a(j) and reduces.
#include "usv_internal.h"

namespace usv {
namespace {

constexpr int kRows = 32;

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// grid = (ceil(nb_valid / 32), B*Hh); 1024 threads (the grid is small, 192 workgroups at the 480p shape, and every
// step is a memory latency: sixteen waves per CU overlap what four cannot).
constexpr int kPartThreads = 1024;
__global__ __launch_bounds__(kPartThreads) void entropy_partials(const float* __restrict__ scores,
                                                                 float* __restrict__ partial, int nb, int nb_valid,
                                                                 int tiles) {
  constexpr int NW = kPartThreads / 64, RPW = kRows / NW;  // 16 waves, 2 rows each
  __shared__ float row_max[kRows], row_inv[kRows];
  __shared__ float upper[kPartThreads / 2];
  const int bh = blockIdx.y, i0 = blockIdx.x * kRows;
  const float* S = scores + (long long)bh * nb * nb;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // row statistics: wave w owns rows RPW w .. +RPW; the loads of its rows of a 512-cube chunk are issued together
  float mx[RPW], sum[RPW];
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) mx[rr] = -INFINITY, sum[rr] = 0.f;
  for (int pass = 0; pass < 2; ++pass) {
    for (int jc = 0; jc < nb_valid; jc += 512) {
      float x[RPW][8];
#pragma unroll
      for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const int i = i0 + wave * RPW + rr, j = jc + 64 * t + lane;
          x[rr][t] = (i < nb_valid && j < nb_valid) ? S[(long long)i * nb + j] : -INFINITY;
        }
#pragma unroll
      for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          if (pass == 0)
            mx[rr] = fmaxf(mx[rr], x[rr][t]);
          else
            sum[rr] += __builtin_amdgcn_exp2f((x[rr][t] - mx[rr]) * kLog2e);  // exp2(-inf) = 0 outside the valid cubes
        }
    }
    if (pass == 0) {
#pragma unroll
      for (int rr = 0; rr < RPW; ++rr) {
        mx[rr] = wave_max(mx[rr]);
        if (mx[rr] == -INFINITY) mx[rr] = 0.f;  // a row of a cube without a valid token: all terms stay 0
      }
    }
  }
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    const float l = wave_sum(sum[rr]);
    if (lane == 0) {
      row_max[wave * RPW + rr] = mx[rr];
      row_inv[wave * RPW + rr] = l > 0.f ? 1.0f / l : 0.f;
    }
  }
  __syncthreads();

  // column sums of the 32 normalised rows: thread (column, half) adds rows 16 half .. +16 in ascending order,
  // then lower half + upper half
  float* dst = partial + ((long long)bh * tiles + blockIdx.x) * nb;
  const int col = tid & (kPartThreads / 2 - 1), half = tid / (kPartThreads / 2);
  for (int j0 = 0; j0 < nb_valid; j0 += kPartThreads / 2) {  // uniform trip count: barriers inside
    const int j = j0 + col;
    float c = 0.f;
    if (j < nb_valid) {
      float x[kRows / 2];
#pragma unroll
      for (int r = 0; r < kRows / 2; ++r) {
        const int i = i0 + half * (kRows / 2) + r;
        x[r] = i < nb_valid ? S[(long long)i * nb + j] : -INFINITY;
      }
#pragma unroll
      for (int r = 0; r < kRows / 2; ++r) {
        const int rl = half * (kRows / 2) + r;
        c += __builtin_amdgcn_exp2f((x[r] - row_max[rl]) * kLog2e) * row_inv[rl];
      }
    }
    if (half == 1) upper[col] = c;
    __syncthreads();
    if (half == 0 && j < nb_valid) dst[j] = c + upper[col];
    __syncthreads();
  }
}

// grid = B; 1024 threads: 256 columns x 4 row groups.  Row group q adds partial rows q, q + 4, ... (eight
// loads in flight), the four group sums are added in a fixed order.
__global__ __launch_bounds__(1024) void entropy_finish(const float* __restrict__ partial, float* __restrict__ entropy,
                                                       int nb, int nb_valid, int Hh, int tiles) {
  __shared__ float grp[4][256];
  __shared__ float red[256];
  const int b = blockIdx.x, tid = threadIdx.x, col = tid & 255, q = tid >> 8;
  const int T = Hh * tiles;
  const float* p = partial + (long long)b * T * nb;
  const float inv_rows = 1.0f / ((float)Hh * (float)nb_valid);
  float acc = 0.f;
  for (int j0 = 0; j0 < nb_valid; j0 += 256) {  // uniform trip count: barriers inside
    const int j = j0 + col;
    float a = 0.f;
    if (j < nb_valid) {
      int t = q;
      for (; t + 28 < T; t += 32) {
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = p[(long long)(t + 4 * u) * nb + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) a += x[u];
      }
      for (; t < T; t += 4) a += p[(long long)t * nb + j];
    }
    grp[q][col] = a;
    __syncthreads();
    if (q == 0 && j < nb_valid) {
      const float m = (((grp[0][col] + grp[1][col]) + grp[2][col]) + grp[3][col]) * inv_rows;
      if (m > 0.f) acc += m * logf(m);
    }
    __syncthreads();
  }
  if (q == 0) red[col] = acc;
  __syncthreads();
  for (int s = 128; s >= 1; s >>= 1) {
    if (tid < s) red[tid] += red[tid + s];
    __syncthreads();
  }
  if (tid == 0) entropy[b] = nb_valid > 1 ? -red[0] / logf((float)nb_valid) : 0.f;
}

}  // namespace

// ws: B * Hh * tiles * nb floats, tiles = ceil(nb_valid / 32)
hipError_t launch_attn_entropy(const float* scores, const Dims& s, float* entropy, float* ws, hipStream_t st) {
  const int tiles = (s.nb_valid + kRows - 1) / kRows;
  entropy_partials<<<dim3((unsigned)tiles, (unsigned)s.bh()), kPartThreads, 0, st>>>(scores, ws, s.nb, s.nb_valid, tiles);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  entropy_finish<<<(unsigned)s.B, 1024, 0, st>>>(ws, entropy, s.nb, s.nb_valid, s.Hh, tiles);
  return hipGetLastError();
}

}  // namespace usv
