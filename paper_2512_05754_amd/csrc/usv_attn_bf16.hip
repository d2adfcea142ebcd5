// Stage 3, bf16 path: block-sparse flash attention on the gfx950 matrix cores
// (masked-attention equation, paper Section 3.2; only listed K/V cubes are touched).
//
// Work decomposition (one workgroup = 4 wavefronts = one 64-row query block):
//   wave (qh, kh): query rows 32*qh .. +32, keys 32*kh .. +32 of every listed 64-key tile.
//   Each wave runs an independent online softmax over its half of the keys; the two key halves
//   are merged once, at the end, through LDS.  All four waves share the K/V tile in LDS, so a
//   tile is fetched from L2/HBM once per query block.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, fp32 accumulate):
//   S^T (32 keys x 32 queries) = K_tile (A operand, rows = keys) x Q^T (B operand, cols = queries)
//   O^T (32 d    x 32 queries) = V^T    (A operand, rows = d)    x P^T (B operand, cols = queries)
// Working on the transposes puts one query per lane column: row max, row sum and the rescale
// factor are per-lane values, and the S^T accumulator registers are, as they stand, the P^T
// operand of the second product (the contraction index of an MFMA can be enumerated in any
// order as long as both operands agree, so V^T is read in the order the accumulator holds keys).
// V^T fragments come from the row-major V tile with the LDS transpose read ds_read_b64_tr_b16.
//
// LDS: double-buffered K and V tiles (2 x 2 x 64 x D bf16), 16-byte chunks XOR-swizzled so that
// both the 16-byte K fragment reads and the transposing V reads spread over all banks.
#include "usv_internal.h"

namespace usv {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4v;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kThreads = 256;

template <int D>
struct Tile {
  static constexpr int kChunks = D / 8;           // 16-byte chunks per row
  static constexpr int kRowBytes = D * 2;
  static constexpr int kBytes = kBlock * D * 2;   // one K or V tile
  static constexpr int kLoads = kBlock * kChunks / kThreads;  // 16-byte loads per thread per tile
  // K: lanes 0..15 of a fragment read hit 16 consecutive rows at one chunk column.
  __device__ static int k_swz(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
  // V: a transposing read touches 8 consecutive rows x 4 consecutive chunks.
  __device__ static int v_swz(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : (((row & 1) << 2) | ((row >> 1) & 3));
  }
  __device__ static int k_off(int row, int chunk) { return row * kRowBytes + ((chunk ^ k_swz(row)) << 4); }
  __device__ static int v_off(int row, int chunk) { return row * kRowBytes + ((chunk ^ v_swz(row)) << 4); }
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float other_half(float x) {  // value held by lane ^ 32
  return __shfl_xor(x, 32);
}

template <int D, bool OUT_F32>
__global__ __launch_bounds__(kThreads, 2) void attn_bf16(const uint16_t* __restrict__ q,
                                                         const uint16_t* __restrict__ k,
                                                         const uint16_t* __restrict__ v,
                                                         const int32_t* __restrict__ idx,
                                                         const int32_t* __restrict__ cnt,
                                                         void* __restrict__ out, float* __restrict__ lse,
                                                         int nb, int Nv, int kmax, float scale_log2e,
                                                         int total, int per_xcd) {
  using T = Tile<D>;
  constexpr int KSTEPS = D / 16;  // MFMA k-steps of the QK^T product
  constexpr int DSUB = D / 32;    // 32-wide d sub-tiles of the output
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * T::kBytes];
  unsigned char* const Kbuf = smem;                  // [2][kBytes]
  unsigned char* const Vbuf = smem + 2 * T::kBytes;  // [2][kBytes]

  const int work = xcd_contiguous_id(blockIdx.x, per_xcd);
  if (work >= total) return;  // whole workgroup leaves before any barrier
  const int i = work % nb;
  const long long head = work / nb;
  const long long head_off = head * (long long)nb * kBlock * D;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int qh = wave & 1, kh = wave >> 1;
  const int col = lane & 31, g = lane >> 5;
  const int n_list = cnt[work];
  const int32_t* list = idx + (long long)work * kmax;

  // Q fragments: lane holds query row 32*qh + col, channels 16 t + 8 g .. + 8 for every k-step t
  bf16x8 qf[KSTEPS];
  {
    const uint16_t* qp = q + head_off + (long long)(i * kBlock + qh * 32 + col) * D + g * 8;
#pragma unroll
    for (int t = 0; t < KSTEPS; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qp + t * 16);
  }

  f32x16 o[DSUB];
#pragma unroll
  for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[ds][r] = 0.f;
  float m = -INFINITY;  // running max of the scaled logits (log2 domain), shared by both lane halves
  float l = 0.f;        // this lane's partial row sum (its 16 keys per tile)

  // global -> register staging of one K and one V tile (kLoads 16-byte pieces each per thread)
  uint4 kst[T::kLoads], vst[T::kLoads];
  auto fetch = [&](int j) {
    const uint16_t* kp = k + head_off + (long long)j * kBlock * D;
    const uint16_t* vp = v + head_off + (long long)j * kBlock * D;
#pragma unroll
    for (int it = 0; it < T::kLoads; ++it) {
      const int id = it * kThreads + tid;
      kst[it] = *reinterpret_cast<const uint4*>(kp + id * 8);
      vst[it] = *reinterpret_cast<const uint4*>(vp + id * 8);
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int it = 0; it < T::kLoads; ++it) {
      const int id = it * kThreads + tid;
      const int row = id / T::kChunks, c = id % T::kChunks;
      *reinterpret_cast<uint4*>(Kbuf + buf * T::kBytes + T::k_off(row, c)) = kst[it];
      *reinterpret_cast<uint4*>(Vbuf + buf * T::kBytes + T::v_off(row, c)) = vst[it];
    }
  };

  if (n_list > 0) {
    fetch(list[0]);
    stash(0);
  }
  __syncthreads();

  for (int n = 0; n < n_list; ++n) {
    const int j = list[n];
    const int buf = n & 1;
    const bool more = n + 1 < n_list;
    if (more) fetch(list[n + 1]);

    // ---- S^T = K Q^T over this wave's 32 keys --------------------------------------------
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
    {
      const unsigned char* kb = Kbuf + buf * T::kBytes;
      const int krow = kh * 32 + col;
#pragma unroll
      for (int t = 0; t < KSTEPS; ++t) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kb + T::k_off(krow, 2 * t + g));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], s, 0, 0, 0);
      }
    }
    // register r of lane (col, g) is key 32 kh + 8 (r/4) + 4 g + (r%4) of the tile, query col
    const int nkeys = Nv - j * kBlock;  // valid keys in this tile (>= 64 except in the last block)
    if (nkeys < kBlock) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = kh * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        if (key >= nkeys) s[r] = -INFINITY;
      }
    }

    // ---- online softmax (log2 domain) -----------------------------------------------------
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    mx = fmaxf(mx, other_half(mx));
    const float m_new = fmaxf(m, mx * scale_log2e);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;  // all keys masked so far
    const float alpha = fast_exp2(m - m_use);
    m = m_new;
    float psum = 0.f;
    bf16x8 pf[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const __bf16 p = (__bf16)fast_exp2(fmaf(s[r], scale_log2e, -m_use));
      // the row sum is taken over the ROUNDED probabilities, the ones P V actually uses, so
      // that the final division cancels the rounding of a dominant key instead of keeping it
      psum += (float)p;
      pf[r >> 3][r & 7] = p;
    }
    l = fmaf(l, alpha, psum);
#pragma unroll
    for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[ds][r] *= alpha;

    // ---- O^T += V^T P^T ---------------------------------------------------------------------
    {
      const unsigned char* vb = Vbuf + buf * T::kBytes;
      const int l16 = lane & 15;
#pragma unroll
      for (int ds = 0; ds < DSUB; ++ds) {
        // this lane's 16-lane group covers channels dbase .. dbase + 16
        const int dbase = 32 * ds + 16 * ((lane >> 4) & 1);
        const int dcol = dbase + 4 * (l16 & 3);       // 4 channels = half a 16-byte chunk
        const int chunk = dcol >> 3, half = (dcol >> 2) & 1;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          // keys 16 t + 4 g + (0..3) and 16 t + 8 + 4 g + (0..3) of this wave's half
          const int key0 = kh * 32 + 16 * t + 4 * g + (l16 >> 2);
          const int key1 = key0 + 8;
          const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (short4v __attribute__((address_space(3)))*)(vb + T::v_off(key0, chunk) + half * 8));
          const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (short4v __attribute__((address_space(3)))*)(vb + T::v_off(key1, chunk) + half * 8));
          typedef __attribute__((__vector_size__(8 * sizeof(short)))) short short8v;
          const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          bf16x8 vf;
          __builtin_memcpy(&vf, &both, sizeof(vf));
          o[ds] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[t], o[ds], 0, 0, 0);
        }
      }
    }

    if (more) stash(buf ^ 1);
    __syncthreads();
  }

  // ---- merge the two key halves and write out --------------------------------------------
  // (the last loop iteration ended with a barrier, so the tile buffers are free to reuse)
  const float l_row = l + other_half(l);
  float* xch = reinterpret_cast<float*>(smem);  // [2 qh][DSUB*16 + 2][64 lanes]
  constexpr int XROWS = DSUB * 16 + 2;
  if (kh == 1) {
    float* dst = xch + (qh * XROWS) * 64 + lane;
#pragma unroll
    for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
      for (int r = 0; r < 16; ++r) dst[(ds * 16 + r) * 64] = o[ds][r];
    dst[(DSUB * 16) * 64] = m;
    dst[(DSUB * 16 + 1) * 64] = l_row;
  }
  __syncthreads();
  if (kh == 0) {
    const float* src = xch + (qh * XROWS) * 64 + lane;
    const float m1 = src[(DSUB * 16) * 64], l1 = src[(DSUB * 16 + 1) * 64];
    const float mm = fmaxf(m, m1);
    const float m_use = mm == -INFINITY ? 0.f : mm;
    const float a0 = fast_exp2(m - m_use), a1 = fast_exp2(m1 - m_use);
    const float lt = l_row * a0 + l1 * a1;
    const int token = i * kBlock + qh * 32 + col;
    const bool live = token < Nv && n_list > 0;
    const float inv = live ? 1.f / lt : 0.f;
    const float w0 = a0 * inv, w1 = a1 * inv;
    const long long row_off = head_off + (long long)token * D;
#pragma unroll
    for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        float val[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = rq * 4 + e;
          val[e] = live ? o[ds][r] * w0 + src[(ds * 16 + r) * 64] * w1 : 0.f;
        }
        // register r = 4 rq + e is channel 32 ds + 8 rq + 4 g + e
        const int ch = 32 * ds + 8 * rq + 4 * g;
        if (OUT_F32) {
          *reinterpret_cast<float4*>(static_cast<float*>(out) + row_off + ch) =
              make_float4(val[0], val[1], val[2], val[3]);
        } else {
          bf16x4 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk[e] = (__bf16)val[e];
          *reinterpret_cast<bf16x4*>(static_cast<uint16_t*>(out) + row_off + ch) = pk;
        }
      }
    if (lse && g == 0) lse[head * (long long)nb * kBlock + token] = live ? (mm + __log2f(lt)) * kLn2 : -INFINITY;
  }
}


template <int D, bool OUT_F32>
hipError_t run(const void* q, const void* k, const void* v, const Dims& s, const int32_t* idx, const int32_t* cnt,
               int kmax, float scale, void* out, float* lse, hipStream_t st) {
  const long long total = s.bh() * s.nb;
  const int per_xcd = (int)((total + kNumXcd - 1) / kNumXcd);
  const unsigned grid = (unsigned)per_xcd * kNumXcd;
  const float sl2 = scale * kLog2e;
  auto Q = static_cast<const uint16_t*>(q);
  auto K = static_cast<const uint16_t*>(k);
  auto V = static_cast<const uint16_t*>(v);
  attn_bf16<D, OUT_F32><<<grid, kThreads, 0, st>>>(Q, K, V, idx, cnt, out, lse, s.nb, s.Nv, kmax, sl2, (int)total,
                                                    per_xcd);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_bf16(const void* q, const void* k, const void* v, const Dims& s, const int32_t* idx,
                            const int32_t* cnt, int kmax, float scale, void* out, bool out_f32, float* lse,
                            hipStream_t st) {
  if (s.d == 128)
    return out_f32 ? run<128, true>(q, k, v, s, idx, cnt, kmax, scale, out, lse, st)
                   : run<128, false>(q, k, v, s, idx, cnt, kmax, scale, out, lse, st);
  return out_f32 ? run<64, true>(q, k, v, s, idx, cnt, kmax, scale, out, lse, st)
                 : run<64, false>(q, k, v, s, idx, cnt, kmax, scale, out, lse, st);
}

}  // namespace usv
