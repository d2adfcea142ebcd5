// Stage 3, fp32 variant: block-sparse attention for fp32 Q/K/V in fp32 arithmetic throughout
// (masked-attention equation, paper Section 3.2).  This is the accuracy path (inputs that must
// match an fp64 evaluation to 1e-5); the throughput path is the bf16 kernel.
//
// Same decomposition as the bf16 kernel: one workgroup = 4 wavefronts = one 64-row query block,
// wave (qh, kh) = 32 queries x 32 keys of every listed 64-key tile, an online softmax per key
// half, the two halves merged once at the end through LDS.  Both products run on the fp32 matrix
// cores (v_mfma_f32_32x32x2_f32: fp32 operands, fp32 accumulation), on the transposes:
//   S^T (32 keys x 32 queries) = K (A operand) x Q^T (B operand)
//   O^T (32 d    x 32 queries) = V^T (A operand) x P^T (B operand)
// so that one query sits in one lane column and max / sum / rescale are per-lane values.  An MFMA
// step contracts two indices, one per 32-lane half g.  Which two is free as long as both operands
// agree: in the first product half g takes channels g*D/2 + t at step t (every lane reads its
// operands as contiguous 16-byte pieces), in the second the step r takes, in half g, exactly the
// key that accumulator register r of that half holds, so P^T needs no data movement at all.
// K and V tiles are staged in LDS as fp32 (rows padded by 4 floats), single-buffered: the kernel is
// bound by the fp32 matrix pipe (128 MFMAs of 64 clocks per wave and tile), not by the staging.
#include "usv_internal.h"

namespace usv {
namespace {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// Lanes l and l ^ 32 hold the two key quarters of one query: (value of the low lane, of the high lane) in both.
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  lo = __uint_as_float(r[0]);
  hi = __uint_as_float(r[1]);
}

template <int D>
__global__ __launch_bounds__(256) void attn_f32(const float* __restrict__ q, const float* __restrict__ k,
                                                const float* __restrict__ v, const int32_t* __restrict__ idx,
                                                const int32_t* __restrict__ cnt, float* __restrict__ out,
                                                float* __restrict__ lse, int nb, int Nv, int kmax, float scale_log2e) {
  constexpr int LD = D + 4;      // LDS row stride in floats: 16-byte reads of consecutive rows spread over the banks
  constexpr int DSUB = D / 32;   // 32-wide d sub-tiles of the output
  constexpr int HALF = D / 2;    // channels per lane half in the first product
  constexpr int XROWS = DSUB * 16 + 2;  // exchange rows per wave: O registers, m, l
  static_assert(2 * XROWS * 64 == kBlock * LD, "the exchange area of the two query halves fills the K tile exactly");
  __shared__ __attribute__((aligned(16))) float Ks[kBlock * LD];  // K tile; at the end the exchange area
  __shared__ __attribute__((aligned(16))) float Vs[kBlock * LD];  // V tile; at the end the output staging rows

  const long long blk = blockIdx.x;  // (b*Hh + h) * nb + i
  const int i = (int)(blk % nb);
  const long long head = blk / nb;
  const long long head_off = head * (long long)nb * kBlock * D;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qh = wave & 1, kh = wave >> 1;
  const int col = lane & 31, g = lane >> 5;
  const int n_list = min(max(cnt[blk], 0), kmax);  // device contents are not trusted with addresses

  // Q fragments: lane (col, g) holds channels g*HALF .. +HALF of query row 32 qh + col
  float qf[HALF];
  {
    const float* qp = q + head_off + (long long)(i * kBlock + qh * 32 + col) * D + g * HALF;
#pragma unroll
    for (int e = 0; e < HALF; e += 4) {
      const float4 t = *reinterpret_cast<const float4*>(qp + e);
      qf[e] = t.x; qf[e + 1] = t.y; qf[e + 2] = t.z; qf[e + 3] = t.w;
    }
  }
  f32x16 o[DSUB];
#pragma unroll
  for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[ds][r] = 0.f;
  float m = -INFINITY;  // running max of this wave's keys (log2 domain), identical in both lane halves
  float l = 0.f;        // this lane's partial row sum

  for (int n = 0; n < n_list; ++n) {
    const int j = min(max(idx[blk * kmax + n], 0), nb - 1);
    __syncthreads();  // the previous tile is fully consumed
    {
      const float* kp = k + head_off + (long long)j * kBlock * D;
      const float* vp = v + head_off + (long long)j * kBlock * D;
#pragma unroll
      for (int e = tid; e < kBlock * (D / 4); e += 256) {
        const int row = e / (D / 4), c = (e % (D / 4)) * 4;
        *reinterpret_cast<float4*>(Ks + row * LD + c) = *reinterpret_cast<const float4*>(kp + row * D + c);
        *reinterpret_cast<float4*>(Vs + row * LD + c) = *reinterpret_cast<const float4*>(vp + row * D + c);
      }
    }
    __syncthreads();

    // ---- S^T = K Q^T over this wave's 32 keys -------------------------------------------------
    // Four accumulators, a quarter of the channel steps each, added at the end: the logits reach several
    // hundred before scaling, and a single 64-step fp32 chain rounds them too coarsely for the 1e-5 bound.
    f32x16 s;
    {
      f32x16 sp[4];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) sp[a][r] = 0.f;
      const float* kr = Ks + (kh * 32 + col) * LD + g * HALF;
#pragma unroll
      for (int t = 0; t < HALF; t += 4) {
        const int a = t / (HALF / 4);
        const float4 kv = *reinterpret_cast<const float4*>(kr + t);
        sp[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(kv.x, qf[t], sp[a], 0, 0, 0);
        sp[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(kv.y, qf[t + 1], sp[a], 0, 0, 0);
        sp[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(kv.z, qf[t + 2], sp[a], 0, 0, 0);
        sp[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(kv.w, qf[t + 3], sp[a], 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = (sp[0][r] + sp[1][r]) + (sp[2][r] + sp[3][r]);
    }
    // register r of lane (col, g) is key 32 kh + 8 (r/4) + 4 g + (r%4) of the tile, query col
    const int nkeys = Nv - j * kBlock;  // valid keys of the tile (>= 64 except in the last, partial block)
    if (nkeys < kBlock) {
      const int lim = nkeys - (kh * 32 + 4 * g);
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = (8 * (r >> 2) + (r & 3)) < lim ? s[r] : -INFINITY;
    }

    // ---- online softmax (log2 domain) ---------------------------------------------------------
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    {
      float lo, hi;
      both_halves(mx, lo, hi);
      mx = fmaxf(lo, hi) * scale_log2e;
    }
    const float m_new = fmaxf(m, mx);
    const float m_ref = m_new == -INFINITY ? 0.f : m_new;  // every key so far masked: all p are exp2(-inf) = 0
    if (__any(m_new > m)) {  // wave-uniform; rows whose max did not move get alpha = 1
      const float alpha = __builtin_amdgcn_exp2f(m - m_ref);  // m = -inf -> 0
      l *= alpha;
#pragma unroll
      for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[ds][r] *= alpha;
    }
    m = m_new;
    float p[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2e, -m_ref));
      l += p[r];
    }

    // ---- O^T += V^T P^T: step r contracts, in half g, the key that register r of that half holds ----
    {
      const float* vr = Vs + (kh * 32 + 4 * g) * LD + col;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float* vk = vr + (8 * (r >> 2) + (r & 3)) * LD;
#pragma unroll
        for (int ds = 0; ds < DSUB; ++ds) o[ds] = __builtin_amdgcn_mfma_f32_32x32x2f32(vk[32 * ds], p[r], o[ds], 0, 0, 0);
      }
    }
  }

  // ---- merge the two key halves, stage the block row-major, store coalesced -------------------
  __syncthreads();  // every wave is done with the last tile: Ks and Vs are free
  float l_lo, l_hi;
  both_halves(l, l_lo, l_hi);
  const float l_row = l_lo + l_hi;
  float* xch = Ks + qh * XROWS * 64;  // [XROWS][64 lanes] of this query half
  if (kh == 1) {
    float* dst = xch + lane;
#pragma unroll
    for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
      for (int r = 0; r < 16; ++r) dst[(ds * 16 + r) * 64] = o[ds][r];
    dst[(DSUB * 16) * 64] = m;
    dst[(DSUB * 16 + 1) * 64] = l_row;
  }
  __syncthreads();
  if (kh == 0) {
    const float* src = xch + lane;
    const float m1 = src[(DSUB * 16) * 64], l1 = src[(DSUB * 16 + 1) * 64];
    const float mm = fmaxf(m, m1);
    const float m_ref = mm == -INFINITY ? 0.f : mm;
    const float a0 = __builtin_amdgcn_exp2f(m - m_ref), a1 = __builtin_amdgcn_exp2f(m1 - m_ref);
    const float lt = l_row * a0 + l1 * a1;
    const int token = i * kBlock + qh * 32 + col;
    const bool live = token < Nv && n_list > 0 && lt > 0.f;
    const float inv = live ? 1.f / lt : 0.f;
    const float w0 = live ? a0 * inv : 0.f, w1 = live ? a1 * inv : 0.f;
    float* stage = Vs + (qh * 32 + col) * LD;  // row (32 qh + col) of the block
#pragma unroll
    for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {  // register r = 4 rq + e is channel 32 ds + 8 rq + 4 g + e
        float4 val;
        val.x = live ? o[ds][rq * 4] * w0 + src[(ds * 16 + rq * 4) * 64] * w1 : 0.f;
        val.y = live ? o[ds][rq * 4 + 1] * w0 + src[(ds * 16 + rq * 4 + 1) * 64] * w1 : 0.f;
        val.z = live ? o[ds][rq * 4 + 2] * w0 + src[(ds * 16 + rq * 4 + 2) * 64] * w1 : 0.f;
        val.w = live ? o[ds][rq * 4 + 3] * w0 + src[(ds * 16 + rq * 4 + 3) * 64] * w1 : 0.f;
        *reinterpret_cast<float4*>(stage + 32 * ds + 8 * rq + 4 * g) = val;
      }
    if (lse && g == 0) lse[head * (long long)nb * kBlock + token] = live ? (mm + __log2f(lt)) * kLn2 : -INFINITY;
  }
  __syncthreads();
  {
    // 64 rows x D channels, 4 channels per thread per pass, consecutive threads -> consecutive addresses
    float* ob = out + head_off + (long long)i * kBlock * D;
#pragma unroll
    for (int e = tid; e < kBlock * (D / 4); e += 256) {
      const int row = e / (D / 4), c = (e % (D / 4)) * 4;
      *reinterpret_cast<float4*>(ob + row * D + c) = *reinterpret_cast<const float4*>(Vs + row * LD + c);
    }
  }
}

}  // namespace

hipError_t launch_attn_f32(const float* q, const float* k, const float* v, const Dims& s, const int32_t* idx,
                           const int32_t* cnt, int kmax, float scale, float* out, float* lse, hipStream_t st) {
  const unsigned grid = (unsigned)(s.bh() * s.nb);
  const float sl2 = scale * kLog2e;
  if (s.d == 128)
    attn_f32<128><<<grid, 256, 0, st>>>(q, k, v, idx, cnt, out, lse, s.nb, s.Nv, kmax, sl2);
  else
    attn_f32<64><<<grid, 256, 0, st>>>(q, k, v, idx, cnt, out, lse, s.nb, s.Nv, kmax, sl2);
  return hipGetLastError();
}

}  // namespace usv
