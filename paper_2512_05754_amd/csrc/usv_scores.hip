// Stage 1: pooled block scores (coarse stage of the coarse-to-fine sparse attention,
// paper Sections 2.2 and 3.2).  Two kernels:
//   pool_means   HBM-bound: reads Q and K once with 16-byte coalesced loads, reduces each
//                64-token cube to its fp32 mean over the valid tokens.
//   score_gemm   S = Qm Km^T / sqrt(d) per head on the fp32 matrix cores (fp32 operands and
//                accumulation: the scores keep fp32 accuracy; bf16 MFMA would not).
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
    // streaming read: nothing in this kernel touches a row twice (2.5 us of 50 at the 480p shape)
    typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u4;
    const u4 vv = __builtin_nontemporal_load(reinterpret_cast<const u4*>(p));
    const uint4 v = make_uint4(vv[0], vv[1], vv[2], vv[3]);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

// grid = (B*Hh*nb, 2); blockIdx.y selects Q (0) or K (1).  One workgroup per cube.
// RASTER: the tensors are in raster token order; row r of cube i is token ras.order[64 i + r].
template <typename T, int D, bool RASTER = false>
__global__ __launch_bounds__(kPoolThreads) void pool_means(const T* __restrict__ q, const T* __restrict__ k,
                                                           float* __restrict__ ws, int nb, int Nv,
                                                           long long mean_elems_per_tensor, RasterArgs ras = RasterArgs{}) {
  constexpr int VEC = Vec16<T>::kElems;
  constexpr int LPR = D / VEC;              // lanes per token row
  constexpr int RPI = kPoolThreads / LPR;   // rows per iteration
  constexpr int ITERS = kBlock / RPI;
  __shared__ float part[RPI][D + 4];

  const long long blk = blockIdx.x;         // (b*Hh + h) * nb + i
  const int i = (int)(blk % nb);
  const T* src = (blockIdx.y == 0 ? q : k) + blk * (long long)kBlock * D;
  const unsigned char* rbase = nullptr;
  if constexpr (RASTER) {
    const long long bh = blk / nb, b = bh / ras.Hh, h = bh - b * ras.Hh;
    rbase = reinterpret_cast<const unsigned char*>(blockIdx.y == 0 ? q : k) + b * ras.batch + h * ras.head;
  }
  float* dst = ws + (long long)blockIdx.y * mean_elems_per_tensor + blk * D;
  int nvalid = min(kBlock, max(0, Nv - i * kBlock));
  if constexpr (RASTER)
    if (ras.block_valid) nvalid = min(kBlock, max(0, ras.block_valid[i]));

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
      if constexpr (RASTER)
        Vec16<T>::load(reinterpret_cast<const T*>(rbase + (long long)ras.order[i * kBlock + r] * ras.tok) + c0, x);
      else
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

// S[bh, i, j] = sum_c Qm[bh,i,c] Km[bh,j,c] * rsqrt_d on the fp32 matrix cores
// (v_mfma_f32_32x32x2_f32: fp32 operands and accumulation, so the scores keep fp32 accuracy).
// 64x64 output tile per workgroup, one 32x32 quadrant per wave; the pooled means are staged in LDS
// 64 channels at a time.  An MFMA step contracts 2 channels, one per 32-lane half; which channels a
// step takes is free as long as both operands agree, so half g takes channels 32 g + t at step t
// and every lane reads its operands as contiguous 16-byte pieces.
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

template <int D>
__global__ __launch_bounds__(256) void score_gemm(const float* __restrict__ qm, const float* __restrict__ km,
                                                  float* __restrict__ scores, int nb, int nb_valid,
                                                  float rsqrt_d) {
  constexpr int KC = 64;        // channels staged per pass
  constexpr int LD = KC + 4;    // row stride in floats: 16-byte reads of 32 consecutive rows spread over the banks
  __shared__ __attribute__((aligned(16))) float As[64 * LD];
  __shared__ __attribute__((aligned(16))) float Bs[64 * LD];
  const int bh = blockIdx.z;
  const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const float* qbase = qm + (long long)bh * nb * D;
  const float* kbase = km + (long long)bh * nb * D;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;  // this wave's quadrant
  const int r = lane & 31, g = lane >> 5;
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  // each thread stages 4 + 4 float4 per pass; the next pass's loads are issued before this pass's MFMAs
  constexpr int PER = 64 * (KC / 4) / 256;
  float4 ra[PER], rb[PER];
  auto fetch = [&](int kc) {
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int e = tid + u * 256, row = e / (KC / 4), c = (e % (KC / 4)) * 4;
      ra[u] = make_float4(0.f, 0.f, 0.f, 0.f);  // zero rows beyond nb
      rb[u] = ra[u];
      if (i0 + row < nb) ra[u] = *reinterpret_cast<const float4*>(qbase + (long long)(i0 + row) * D + kc + c);
      if (j0 + row < nb) rb[u] = *reinterpret_cast<const float4*>(kbase + (long long)(j0 + row) * D + kc + c);
    }
  };
  fetch(0);
  for (int kc = 0; kc < D; kc += KC) {
    if (kc) __syncthreads();
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int e = tid + u * 256, row = e / (KC / 4), c = (e % (KC / 4)) * 4;
      *reinterpret_cast<float4*>(As + row * LD + c) = ra[u];
      *reinterpret_cast<float4*>(Bs + row * LD + c) = rb[u];
    }
    __syncthreads();
    if (kc + KC < D) fetch(kc + KC);
    const float* ap = As + (wi + r) * LD + 32 * g;
    const float* bp = Bs + (wj + r) * LD + 32 * g;
#pragma unroll
    for (int t = 0; t < 32; t += 4) {
      const float4 a = *reinterpret_cast<const float4*>(ap + t);
      const float4 b = *reinterpret_cast<const float4*>(bp + t);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
    }
  }
  // accumulator register e of lane (r, g): row wi + 8 (e/4) + 4 g + (e%4), column wj + r
  float* out = scores + (long long)bh * nb * nb;
  const int j = j0 + wj + r;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int i = i0 + wi + 8 * (e >> 2) + 4 * g + (e & 3);
    if (i < nb && j < nb) out[(long long)i * nb + j] = (i < nb_valid && j < nb_valid) ? acc[e] * rsqrt_d : -INFINITY;
  }
}

template <typename T, int D>
hipError_t run(const void* q, const void* k, const Dims& s, float* scores, float* ws, hipStream_t st,
               const RasterArgs* ras = nullptr) {
  const long long cubes = s.bh() * s.nb;
  const long long mean_elems = cubes * D;
  if (ras)
    pool_means<T, D, true><<<dim3((unsigned)cubes, 2), kPoolThreads, 0, st>>>(
        static_cast<const T*>(q), static_cast<const T*>(k), ws, s.nb, s.Nv, mean_elems, *ras);
  else
    pool_means<T, D><<<dim3((unsigned)cubes, 2), kPoolThreads, 0, st>>>(
        static_cast<const T*>(q), static_cast<const T*>(k), ws, s.nb, s.Nv, mean_elems);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int tiles = (s.nb + 63) / 64;
  score_gemm<D><<<dim3(tiles, tiles, (unsigned)s.bh()), 256, 0, st>>>(ws, ws + mean_elems, scores, s.nb,
                                                                         s.nb_valid, 1.0f / sqrtf((float)D));
  return hipGetLastError();
}

template <typename T, int D>
hipError_t run_pool(const void* x, const Dims& s, float* means, hipStream_t st, const RasterArgs* ras) {
  const long long cubes = s.bh() * s.nb;
  if (ras)
    pool_means<T, D, true><<<dim3((unsigned)cubes, 1), kPoolThreads, 0, st>>>(
        static_cast<const T*>(x), static_cast<const T*>(x), means, s.nb, s.Nv, cubes * D, *ras);
  else
    pool_means<T, D><<<dim3((unsigned)cubes, 1), kPoolThreads, 0, st>>>(static_cast<const T*>(x), static_cast<const T*>(x),
                                                                        means, s.nb, s.Nv, cubes * D);
  return hipGetLastError();
}

}  // namespace

// Pooled fp32 means of ONE tensor [B, Hh, N, d] -> means [B, Hh, nb, d].
hipError_t launch_pool_means(const void* x, const Dims& s, float* means, hipStream_t st, const RasterArgs* ras) {
  if (s.bf16)
    return s.d == 128 ? run_pool<uint16_t, 128>(x, s, means, st, ras) : run_pool<uint16_t, 64>(x, s, means, st, ras);
  return s.d == 128 ? run_pool<float, 128>(x, s, means, st, ras) : run_pool<float, 64>(x, s, means, st, ras);
}

hipError_t launch_block_scores(const void* q, const void* k, const Dims& s, float* scores, float* ws,
                               hipStream_t st, const RasterArgs* ras) {
  if (s.bf16)
    return s.d == 128 ? run<uint16_t, 128>(q, k, s, scores, ws, st, ras) : run<uint16_t, 64>(q, k, s, scores, ws, st, ras);
  return s.d == 128 ? run<float, 128>(q, k, s, scores, ws, st, ras) : run<float, 64>(q, k, s, scores, ws, st, ras);
}

}  // namespace usv
