// Stage 3, fp32 variant: block-sparse attention for fp32 Q/K/V entirely in fp32 FMA arithmetic
// (masked-attention equation, paper Section 3.2).  This is the accuracy path (inputs that must
// match an fp64 evaluation to 1e-5); the throughput path is the bf16 MFMA kernel.
//
// One workgroup (256 threads) per query block.  Four lanes share one query row, each owning a
// quarter of the head dimension of q and of the output accumulator; K and V tiles of the listed
// blocks are staged in LDS as fp32 and walked key by key with a running-max softmax.
#include "usv_internal.h"

namespace usv {
namespace {

template <int D>
__global__ __launch_bounds__(256) void attn_f32(const float* __restrict__ q, const float* __restrict__ k,
                                                const float* __restrict__ v, const int32_t* __restrict__ idx,
                                                const int32_t* __restrict__ cnt, float* __restrict__ out,
                                                float* __restrict__ lse, int nb, int Nv, int kmax, float scale) {
  constexpr int DP = D / 4;  // channels per lane
  __shared__ float Ks[kBlock * D];
  __shared__ float Vs[kBlock * D];

  const long long blk = blockIdx.x;  // (b*Hh + h) * nb + i
  const int i = (int)(blk % nb);
  const long long head = blk / nb;
  const long long head_off = head * (long long)nb * kBlock * D;
  const int tid = threadIdx.x;
  const int r = tid >> 2, part = tid & 3;
  const int token = i * kBlock + r;
  const int n_list = min(max(cnt[blk], 0), kmax);  // device contents are not trusted with addresses

  float qr[DP], o[DP];
  {
    const float* qp = q + head_off + (long long)token * D + part * DP;
#pragma unroll
    for (int e = 0; e < DP; e += 4) {
      const float4 t = *reinterpret_cast<const float4*>(qp + e);
      qr[e] = t.x; qr[e + 1] = t.y; qr[e + 2] = t.z; qr[e + 3] = t.w;
    }
  }
#pragma unroll
  for (int e = 0; e < DP; ++e) o[e] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int n = 0; n < n_list; ++n) {
    const int j = min(max(idx[blk * kmax + n], 0), nb - 1);
    const int nkeys = min(kBlock, Nv - j * kBlock);  // >= 1 for a listed block
    __syncthreads();                                  // previous tile fully consumed
    const float* kp = k + head_off + (long long)j * kBlock * D;
    const float* vp = v + head_off + (long long)j * kBlock * D;
    for (int e = tid * 4; e < kBlock * D; e += 256 * 4) {
      *reinterpret_cast<float4*>(Ks + e) = *reinterpret_cast<const float4*>(kp + e);
      *reinterpret_cast<float4*>(Vs + e) = *reinterpret_cast<const float4*>(vp + e);
    }
    __syncthreads();
    for (int c = 0; c < nkeys; ++c) {
      const float* kr = Ks + c * D + part * DP;
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < DP; ++e) s = fmaf(qr[e], kr[e], s);
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      s *= scale;
      if (s > m) {  // new running maximum: rescale what has been accumulated
        const float a = expf(m - s);  // m = -inf -> 0
        l *= a;
#pragma unroll
        for (int e = 0; e < DP; ++e) o[e] *= a;
        m = s;
      }
      const float p = expf(s - m);
      l += p;
      const float* vr = Vs + c * D + part * DP;
#pragma unroll
      for (int e = 0; e < DP; ++e) o[e] = fmaf(p, vr[e], o[e]);
    }
  }

  const bool live = token < Nv && n_list > 0;
  const float inv = live ? 1.f / l : 0.f;
  float* op = out + head_off + (long long)token * D + part * DP;
#pragma unroll
  for (int e = 0; e < DP; e += 4)
    *reinterpret_cast<float4*>(op + e) = make_float4(o[e] * inv, o[e + 1] * inv, o[e + 2] * inv, o[e + 3] * inv);
  if (lse && part == 0) lse[head * (long long)nb * kBlock + token] = live ? m + logf(l) : -INFINITY;
}

}  // namespace

hipError_t launch_attn_f32(const float* q, const float* k, const float* v, const Dims& s, const int32_t* idx,
                           const int32_t* cnt, int kmax, float scale, float* out, float* lse, hipStream_t st) {
  const unsigned grid = (unsigned)(s.bh() * s.nb);
  if (s.d == 128)
    attn_f32<128><<<grid, 256, 0, st>>>(q, k, v, idx, cnt, out, lse, s.nb, s.Nv, kmax, scale);
  else
    attn_f32<64><<<grid, 256, 0, st>>>(q, k, v, idx, cnt, out, lse, s.nb, s.Nv, kmax, scale);
  return hipGetLastError();
}

}  // namespace usv
