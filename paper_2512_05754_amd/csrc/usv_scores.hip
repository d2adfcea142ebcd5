// Stage 1: pooled block scores (coarse stage of the coarse-to-fine sparse attention,
// paper Sections 2.2 and 3.2).  Two kernels:
//   pool_means   HBM-bound: reads Q and K once with 16-byte coalesced loads, reduces each
//                64-token cube to its fp32 mean over the valid tokens.
//   score_gemm   S = Qm Km^T / sqrt(d) per head in fp32 (LDS-tiled FMA; the contraction is
//                tiny next to the read of Q and K, so it stays off the bf16 matrix cores to
//                keep the scores at fp32 accuracy).
#include "usv_internal.h"

namespace usv {
namespace {

constexpr int kPoolThreads = 256;

template <typename T>
struct Vec16;  // 16 bytes of T
template <>
struct Vec16<float> {
  static constexpr int kElems = 4;
  __device__ static void load(const float* p, float (&out)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  }
};
template <>
struct Vec16<uint16_t> {  // bf16 bit patterns
  static constexpr int kElems = 8;
  __device__ static void load(const uint16_t* p, float (&out)[8]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

// grid = (B*Hh*nb, 2); blockIdx.y selects Q (0) or K (1).  One workgroup per cube.
template <typename T, int D>
__global__ __launch_bounds__(kPoolThreads) void pool_means(const T* __restrict__ q, const T* __restrict__ k,
                                                           float* __restrict__ ws, int nb, int Nv,
                                                           long long mean_elems_per_tensor) {
  constexpr int VEC = Vec16<T>::kElems;
  constexpr int LPR = D / VEC;              // lanes per token row
  constexpr int RPI = kPoolThreads / LPR;   // rows per iteration
  constexpr int ITERS = kBlock / RPI;
  __shared__ float part[RPI][D + 4];

  const long long blk = blockIdx.x;         // (b*Hh + h) * nb + i
  const int i = (int)(blk % nb);
  const T* src = (blockIdx.y == 0 ? q : k) + blk * (long long)kBlock * D;
  float* dst = ws + (long long)blockIdx.y * mean_elems_per_tensor + blk * D;
  const int nvalid = min(kBlock, max(0, Nv - i * kBlock));

  const int tid = threadIdx.x;
  const int r0 = tid / LPR, c0 = (tid % LPR) * VEC;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int r = r0 + it * RPI;
    if (r < nvalid) {
      float x[VEC];
      Vec16<T>::load(src + (long long)r * D + c0, x);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += x[e];
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) part[r0][c0 + e] = acc[e];
  __syncthreads();
  if (tid < D) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < RPI; ++r) s += part[r][tid];
    // a cube with no valid token has no mean; its scores are overwritten with -inf later
    dst[tid] = nvalid > 0 ? s / (float)nvalid : 0.f;
  }
}

// S[bh, i, j] = sum_c Qm[bh,i,c] Km[bh,j,c] * rsqrt_d.  64x64 output tile per workgroup of 256
// threads; thread (ty, tx) owns the 4x4 patch rows ty+16a, cols tx+16b (interleaved so that LDS
// reads of consecutive lanes hit consecutive rows with an odd-ish padded stride).
template <int D>
__global__ __launch_bounds__(256) void score_gemm(const float* __restrict__ qm, const float* __restrict__ km,
                                                  float* __restrict__ scores, int nb, int nb_valid,
                                                  float rsqrt_d) {
  constexpr int KC = 64;        // channels staged per pass
  constexpr int LD = KC + 4;
  __shared__ float As[64 * LD];
  __shared__ float Bs[64 * LD];
  const int bh = blockIdx.z;
  const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const float* qbase = qm + (long long)bh * nb * D;
  const float* kbase = km + (long long)bh * nb * D;
  const int tid = threadIdx.x;
  const int ty = tid / 16, tx = tid % 16;
  float acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;
  for (int kc = 0; kc < D; kc += KC) {
    if (kc) __syncthreads();
    // stage both 64 x KC tiles (zero rows beyond nb)
    for (int e = tid; e < 64 * (KC / 4); e += 256) {
      const int r = e / (KC / 4), c = (e % (KC / 4)) * 4;
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
      if (i0 + r < nb) a = *reinterpret_cast<const float4*>(qbase + (long long)(i0 + r) * D + kc + c);
      if (j0 + r < nb) b = *reinterpret_cast<const float4*>(kbase + (long long)(j0 + r) * D + kc + c);
      *reinterpret_cast<float4*>(As + r * LD + c) = a;
      *reinterpret_cast<float4*>(Bs + r * LD + c) = b;
    }
    __syncthreads();
#pragma unroll 4
    for (int c = 0; c < KC; c += 4) {
      float4 av[4], bv[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) av[a] = *reinterpret_cast<const float4*>(As + (ty + 16 * a) * LD + c);
#pragma unroll
      for (int b = 0; b < 4; ++b) bv[b] = *reinterpret_cast<const float4*>(Bs + (tx + 16 * b) * LD + c);
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          acc[a][b] = fmaf(av[a].x, bv[b].x, acc[a][b]);
          acc[a][b] = fmaf(av[a].y, bv[b].y, acc[a][b]);
          acc[a][b] = fmaf(av[a].z, bv[b].z, acc[a][b]);
          acc[a][b] = fmaf(av[a].w, bv[b].w, acc[a][b]);
        }
    }
  }
  float* out = scores + (long long)bh * nb * nb;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int i = i0 + ty + 16 * a;
    if (i >= nb) continue;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int j = j0 + tx + 16 * b;
      if (j >= nb) continue;
      const bool live = i < nb_valid && j < nb_valid;
      out[(long long)i * nb + j] = live ? acc[a][b] * rsqrt_d : -INFINITY;
    }
  }
}

template <typename T, int D>
hipError_t run(const void* q, const void* k, const Dims& s, float* scores, float* ws, hipStream_t st) {
  const long long cubes = s.bh() * s.nb;
  const long long mean_elems = cubes * D;
  pool_means<T, D><<<dim3((unsigned)cubes, 2), kPoolThreads, 0, st>>>(
      static_cast<const T*>(q), static_cast<const T*>(k), ws, s.nb, s.Nv, mean_elems);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int tiles = (s.nb + 63) / 64;
  score_gemm<D><<<dim3(tiles, tiles, (unsigned)s.bh()), 256, 0, st>>>(ws, ws + mean_elems, scores, s.nb,
                                                                         s.nb_valid, 1.0f / sqrtf((float)D));
  return hipGetLastError();
}

}  // namespace

hipError_t launch_block_scores(const void* q, const void* k, const Dims& s, float* scores, float* ws,
                               hipStream_t st) {
  if (s.bf16) return s.d == 128 ? run<uint16_t, 128>(q, k, s, scores, ws, st) : run<uint16_t, 64>(q, k, s, scores, ws, st);
  return s.d == 128 ? run<float, 128>(q, k, s, scores, ws, st) : run<float, 64>(q, k, s, scores, ws, st);
}

}  // namespace usv
