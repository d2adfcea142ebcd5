// Cube-level branch and output fusion (paper Figure 2, right: the cube-level result is spread over the
// tokens of the grid again and combined with the token-level one; Section 2.2: the coarse level of the
// coarse-to-fine scheme).
//
//   coarse_attn   C[bh, i, :] = sum_j softmax_j(S[bh, i, :])_j * Vm[bh, j, :] over the cubes that hold a
//                 valid token; S are the stage-1 scores, Vm the pooled fp32 means of V.  Two passes over
//                 the 32 score rows of a workgroup: row maxima, then exp, row sums and P Vm on the fp32
//                 matrix cores (v_mfma_f32_32x32x2_f32).
//   fuse_outputs  out[r] = g_fine[r] * fine[r] + g_coarse[r] * C[cube(r)], elementwise: HBM bound.
#include "usv_internal.h"

namespace usv {
namespace {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// grid = (ceil(nb / 32), B*Hh); 8 D threads = 4 (D/32) wavefronts.  Output tile: 32 query cubes x D channels.
// Pass A finds the row maxima; pass B walks the key cubes 64 at a time: it stages P = exp(S - max) and the Vm
// tile in LDS, accumulates the row sums (8 lanes per row), and runs P Vm on the matrix cores.  Wavefront
// (kg, cg) takes key cubes 16 kg .. +16 of every tile and channels 32 cg .. +32, so a workgroup puts four
// (D=64: two) waves on every SIMD of its CU: the grid is small (192 workgroups at the 480p shape) and the
// kernel is bound by exposed latencies, not by bandwidth or the matrix cores.  The four key groups' partial
// tiles are added in a fixed order at the end.
template <int D>
__global__ __launch_bounds__(8 * D) void coarse_attn(const float* __restrict__ scores, const float* __restrict__ vmean,
                                                     float* __restrict__ coarse, int nb, int nb_valid) {
  constexpr int NT = 8 * D;        // threads
  constexpr int NW = NT / 64;      // wavefronts
  constexpr int ROWS = 32;
  constexpr int RPW = ROWS / NW;   // rows per wave in pass A
  constexpr int LD = 64 + 4;       // row stride of the P tile in floats (16-byte reads of 32 consecutive rows spread over the banks)
  constexpr int VLD = D + 4;       // row stride of the Vm tile and of the reduction buffer
  __shared__ __attribute__((aligned(16))) float Ps[ROWS * LD];  // P tile, [query cube][key cube]
  __shared__ __attribute__((aligned(16))) float Vs[64 * VLD];   // Vm tile, [key cube][channel]; later the reduction buffer
  __shared__ float row_max[ROWS], row_inv[ROWS];
  const int bh = blockIdx.y, i0 = blockIdx.x * ROWS;
  const float* S = scores + (long long)bh * nb * nb;
  const float* vm = vmean + (long long)bh * nb * D;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kg = wave & 3, cg = wave >> 2;
  const int srow = (tid >> 3) & 31, spart = tid & 7;  // row statistics (threads 0..255): 8 lanes per row, 8 key cubes each per tile

  // pass A: row maxima.  Wave w owns rows RPW w .. +RPW; the loads of all its rows of a 512-cube chunk
  // are issued together, so a chunk costs one memory latency.
  {
    float mx[RPW];
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) mx[rr] = -INFINITY;
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
        for (int t = 0; t < 8; ++t) mx[rr] = fmaxf(mx[rr], x[rr][t]);
    }
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      float m = mx[rr];
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
      if (lane == 0) row_max[wave * RPW + rr] = m == -INFINITY ? 0.f : m;  // rows of cubes without a valid token: P stays 0
    }
  }
  __syncthreads();

  // pass B: C = P Vm (unnormalised), row sums on the side.  The next tile's scores and Vm rows are
  // fetched into registers while the current tile is in LDS.
  const int r = lane & 31, g = lane >> 5;
  const int kofs = 16 * kg + 8 * g;  // an MFMA step contracts 2 key cubes, one per 32-lane half: key group kg, half g takes cube 16 kg + 8 g + t at step t
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  float l = 0.f;
  constexpr int SPT = ROWS * 64 / NT;       // scores per thread and tile
  constexpr int VPT = 64 * (D / 4) / NT;    // float4 of Vm per thread and tile
  float sreg[SPT];
  float4 vreg[VPT];
  auto fetch = [&](int j0) {
#pragma unroll
    for (int t = 0; t < SPT; ++t) {
      const int e = tid + NT * t, row = e >> 6, col = e & 63, i = i0 + row, j = j0 + col;
      sreg[t] = (i < nb_valid && j < nb_valid) ? S[(long long)i * nb + j] : -INFINITY;
    }
#pragma unroll
    for (int t = 0; t < VPT; ++t) {
      const int e = tid + NT * t, col = e / (D / 4), c = (e % (D / 4)) * 4, j = j0 + col;
      vreg[t] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j < nb_valid) vreg[t] = *reinterpret_cast<const float4*>(vm + (long long)j * D + c);
    }
  };
  fetch(0);
  for (int j0 = 0; j0 < nb_valid; j0 += 64) {
    if (j0) __syncthreads();  // the previous tile has been consumed
#pragma unroll
    for (int t = 0; t < SPT; ++t) {
      const int e = tid + NT * t, row = e >> 6, col = e & 63;
      // exp2(-inf) = 0 covers the entries outside the valid cubes
      Ps[row * LD + col] = __builtin_amdgcn_exp2f((sreg[t] - row_max[row]) * kLog2e);
    }
#pragma unroll
    for (int t = 0; t < VPT; ++t) {
      const int e = tid + NT * t, col = e / (D / 4), c = (e % (D / 4)) * 4;
      *reinterpret_cast<float4*>(Vs + col * VLD + c) = vreg[t];
    }
    __syncthreads();
    if (j0 + 64 < nb_valid) fetch(j0 + 64);
    if (tid < 256) {
#pragma unroll
      for (int t = 0; t < 8; ++t) l += Ps[srow * LD + spart * 8 + t];
    }
    const float* ap = Ps + r * LD + kofs;
    const float* bp = Vs + kofs * VLD + 32 * cg + r;  // operand of step t: Vm[cube kofs + t][channel 32 cg + r]
#pragma unroll
    for (int t = 0; t < 8; t += 4) {
      const float4 a = *reinterpret_cast<const float4*>(ap + t);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, bp[(t + 0) * VLD], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, bp[(t + 1) * VLD], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, bp[(t + 2) * VLD], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, bp[(t + 3) * VLD], acc, 0, 0, 0);
    }
  }
  if (tid < 256) {
    l += __shfl_xor(l, 1);
    l += __shfl_xor(l, 2);
    l += __shfl_xor(l, 4);
    if (spart == 0) row_inv[srow] = l > 0.f ? 1.0f / l : 0.f;
  }
  __syncthreads();  // also: every wave is done reading Vs

  // add the four key groups' partial tiles in group order (deterministic), then normalise and store.
  // accumulator register e of lane (r, g): row 8 (e/4) + 4 g + (e%4), channel 32 cg + r
  float* red = Vs;
  for (int w = 0; w < 4; ++w) {
    if (kg == w) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float* p = red + (8 * (e >> 2) + 4 * g + (e & 3)) * VLD + 32 * cg + r;
        *p = (w == 0 ? 0.f : *p) + acc[e];
      }
    }
    __syncthreads();
  }
  float* out = coarse + (long long)bh * nb * D;
  for (int e = tid; e < ROWS * (D / 4); e += NT) {
    const int row = e / (D / 4), c = (e % (D / 4)) * 4, i = i0 + row;
    if (i < nb) {
      const float inv = i < nb_valid ? row_inv[row] : 0.f;
      const float4 v = *reinterpret_cast<const float4*>(red + row * VLD + c);
      *reinterpret_cast<float4*>(out + (long long)i * D + c) = make_float4(v.x * inv, v.y * inv, v.z * inv, v.w * inv);
    }
  }
}

// ---- fusion --------------------------------------------------------------------------------------
template <typename T>
struct Elem;  // 4 consecutive channels of T <-> float4
template <>
struct Elem<float> {
  __device__ static float4 load(const float* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static void store(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
};
template <>
struct Elem<uint16_t> {  // bf16 bit patterns
  __device__ static float4 load(const uint16_t* p) {
    const uint2 w = *reinterpret_cast<const uint2*>(p);
    return make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                       __uint_as_float(w.y & 0xffff0000u));
  }
  __device__ static void store(uint16_t* p, float4 v) {
    typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
    bf16x4 o;
    o[0] = (__bf16)v.x; o[1] = (__bf16)v.y; o[2] = (__bf16)v.z; o[3] = (__bf16)v.w;  // round to nearest even
    *reinterpret_cast<bf16x4*>(p) = o;
  }
};

// One thread per 4 channels of one token; consecutive threads -> consecutive addresses.
template <typename FT, typename GT, typename OT>
__global__ __launch_bounds__(256) void fuse_outputs(const FT* __restrict__ fine, const float* __restrict__ coarse,
                                                    const GT* __restrict__ gate_fine, const GT* __restrict__ gate_coarse,
                                                    OT* out, int N, int Nv, int d4, long long total4) {
  const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
  if (id >= total4) return;
  const long long token = id / d4;  // (b*Hh + h) * N + r
  const int c = (int)(id - token * d4) * 4;
  const int r = (int)(token % N);
  const long long off = id * 4;
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
  if (r < Nv) {
    const float4 f = Elem<FT>::load(fine + off);
    const float4 cz = *reinterpret_cast<const float4*>(coarse + (token / kBlock) * (long long)(d4 * 4) + c);
    float4 gf = make_float4(1.f, 1.f, 1.f, 1.f), gc = gf;
    if (gate_fine) gf = Elem<GT>::load(gate_fine + off);
    if (gate_coarse) gc = Elem<GT>::load(gate_coarse + off);
    o.x = fmaf(gf.x, f.x, gc.x * cz.x);
    o.y = fmaf(gf.y, f.y, gc.y * cz.y);
    o.z = fmaf(gf.z, f.z, gc.z * cz.z);
    o.w = fmaf(gf.w, f.w, gc.w * cz.w);
  }
  Elem<OT>::store(out + off, o);
}

template <typename FT, typename GT, typename OT>
hipError_t run_fuse(const void* fine, const float* coarse, const void* gf, const void* gc, void* out, const Dims& s,
                    hipStream_t st) {
  const long long total4 = s.bh() * s.N * (s.d / 4);
  fuse_outputs<FT, GT, OT><<<(unsigned)((total4 + 255) / 256), 256, 0, st>>>(
      static_cast<const FT*>(fine), coarse, static_cast<const GT*>(gf), static_cast<const GT*>(gc), static_cast<OT*>(out),
      s.N, s.Nv, s.d / 4, total4);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_coarse_attn(const float* scores, const float* vmean, const Dims& s, float* coarse, hipStream_t st) {
  const dim3 grid((unsigned)((s.nb + 31) / 32), (unsigned)s.bh());
  if (s.d == 128)
    coarse_attn<128><<<grid, 8 * 128, 0, st>>>(scores, vmean, coarse, s.nb, s.nb_valid);
  else
    coarse_attn<64><<<grid, 8 * 64, 0, st>>>(scores, vmean, coarse, s.nb, s.nb_valid);
  return hipGetLastError();
}

// (b*Hh + h) * N + r must fit the token arithmetic above: N <= 2^18, bh <= 65535.
hipError_t launch_fuse_outputs(const void* fine, bool fine_f32, const float* coarse, const void* gate_fine,
                               const void* gate_coarse, bool gates_f32, void* out, bool out_f32, const Dims& s,
                               hipStream_t st) {
#define USV_FUSE(FT, GT, OT) return run_fuse<FT, GT, OT>(fine, coarse, gate_fine, gate_coarse, out, s, st)
  if (fine_f32) {
    if (gates_f32) {
      if (out_f32) USV_FUSE(float, float, float);
      USV_FUSE(float, float, uint16_t);
    }
    if (out_f32) USV_FUSE(float, uint16_t, float);
    USV_FUSE(float, uint16_t, uint16_t);
  }
  if (gates_f32) {
    if (out_f32) USV_FUSE(uint16_t, float, float);
    USV_FUSE(uint16_t, float, uint16_t);
  }
  if (out_f32) USV_FUSE(uint16_t, uint16_t, float);
  USV_FUSE(uint16_t, uint16_t, uint16_t);
#undef USV_FUSE
}

}  // namespace usv
