// Token merging (paper Section 3.3): 3-D bipartite partition of the raster token grid into merge
// blocks with one destination each, head-averaged key descriptors, cosine similarity of every source
// to its block's destination, the r most similar sources merged into their destinations by mean
// aggregation, the merged sequence [unmerged sources || destinations], and the exact unmerge.
//
//   merge_descriptors  HBM bound: reads K once, m[b,i,:] = mean over heads (fp32) and |m|^2
//   merge_similarity   u[b,i] = cos(m_i, m_dst(i)); -inf at destinations; also blk[i], the rank of
//                      token i's block among the destinations (bit 31 marks the destination)
//   merge_select       one workgroup per batch element: bit-by-bit search for the r-th largest
//                      source key (keys in registers), then one ordered sweep that ranks ties by
//                      index and assigns the rows of the merged sequence (scans, no atomics)
//   merge_rows         merged features: a destination row is the mean of itself and its merged
//                      sources (found by scanning its own block), other rows are copies
//   unmerge_rows       gather: token k reads row row_of[k]
#include "usv_internal.h"

#ifndef USV_MERGE_DESC_HEADS
#define USV_MERGE_DESC_HEADS 12  // heads whose pieces merge_descriptors keeps in flight
#endif
#ifndef USV_MERGE_COPY_ROWS
#define USV_MERGE_COPY_ROWS 2  // rows a lane group copies in usv_merge_apply
#endif

namespace usv {
namespace {

// raster index -> coordinates, destination of the block, rank of a destination among destinations
struct Tok {
  int t, h, w;
};
__device__ __forceinline__ Tok coords(const MergeGrid& g, int i) {
  const int hw = g.H * g.W;
  Tok c;
  c.t = i / hw;
  const int rem = i - c.t * hw;
  c.h = rem / g.W;
  c.w = rem - c.h * g.W;
  return c;
}
__device__ __forceinline__ int dst_index(const MergeGrid& g, const Tok& c) {
  return ((c.t - c.t % g.st) * g.H + (c.h - c.h % g.sh)) * g.W + (c.w - c.w % g.sw);
}
__device__ __forceinline__ bool is_dst(const MergeGrid& g, const Tok& c) {
  return c.t % g.st == 0 && c.h % g.sh == 0 && c.w % g.sw == 0;
}
// destinations in ascending raster order = ascending (t/st, h/sh, w/sw)
__device__ __forceinline__ int dst_rank(const MergeGrid& g, const Tok& c) {
  return ((c.t / g.st) * g.nH + c.h / g.sh) * g.nW + c.w / g.sw;
}

template <typename T>
struct Row;  // 16 bytes of a row <-> floats
template <>
struct Row<float> {
  static constexpr int kElems = 4;
  __device__ static void load(const float* p, float (&o)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
  __device__ static void store(float* p, const float (&o)[4]) { *reinterpret_cast<float4*>(p) = make_float4(o[0], o[1], o[2], o[3]); }
};
template <>
struct Row<uint16_t> {
  static constexpr int kElems = 8;
  __device__ static void load(const uint16_t* p, float (&o)[8]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static void store(uint16_t* p, const float (&o)[8]) {
    typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (__bf16)o[i];  // round to nearest even
    *reinterpret_cast<bf16x8*>(p) = v;
  }
};

typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned chunk_t;  // 16 bytes

// 16 bytes of a row as they lie in memory -> floats
template <typename T>
__device__ __forceinline__ void widen(const chunk_t& c, float (&o)[Row<T>::kElems]);
template <>
__device__ __forceinline__ void widen<float>(const chunk_t& c, float (&o)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = __uint_as_float(c[i]);
}
template <>
__device__ __forceinline__ void widen<uint16_t>(const chunk_t& c, float (&o)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o[2 * i] = __uint_as_float(c[i] << 16);
    o[2 * i + 1] = __uint_as_float(c[i] & 0xffff0000u);
  }
}

// grid = (ceil(N / rows_per_wg), B); a group of LPR lanes owns one token.
template <typename T, int D>
__global__ __launch_bounds__(256) void merge_descriptors(const T* __restrict__ k, float* __restrict__ m,
                                                         float* __restrict__ norm2, int N, int Hh) {
  constexpr int VEC = Row<T>::kElems, LPR = D / VEC, RPW = 256 / LPR;
  const int b = blockIdx.y, row = blockIdx.x * RPW + threadIdx.x / LPR, c0 = (threadIdx.x % LPR) * VEC;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  if (row < N) {
    const T* src = k + ((long long)b * Hh * N + row) * D + c0;
    const long long hs = (long long)N * D;
    int h = 0;
    // that many heads in flight, as raw 16-byte pieces; streaming reads (nothing here touches a byte of K twice, and a
    // read that leaves its lines in the caches costs this kernel a third of its time: 30 -> 21 us at 480p)
    for (; h + USV_MERGE_DESC_HEADS <= Hh; h += USV_MERGE_DESC_HEADS) {
      chunk_t raw[USV_MERGE_DESC_HEADS];
#pragma unroll
      for (int u = 0; u < USV_MERGE_DESC_HEADS; ++u) raw[u] = __builtin_nontemporal_load(reinterpret_cast<const chunk_t*>(src + (h + u) * hs));
#pragma unroll
      for (int u = 0; u < USV_MERGE_DESC_HEADS; ++u) {  // ascending heads: the order of the additions does not depend on the batch
        float xv[VEC];
        widen<T>(raw[u], xv);
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += xv[e];
      }
    }
    for (; h < Hh; ++h) {
      float x[VEC];
      Row<T>::load(src + h * hs, x);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += x[e];
    }
  }
  const float inv = 1.0f / (float)Hh;
  float n2 = 0.f;
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    acc[e] *= inv;
    n2 = fmaf(acc[e], acc[e], n2);
  }
#pragma unroll
  for (int o = LPR / 2; o >= 1; o >>= 1) n2 += __shfl_xor(n2, o);  // LPR <= 32 consecutive lanes of one wave
  if (row < N) {
    float* dst = m + ((long long)b * N + row) * D + c0;
#pragma unroll
    for (int e = 0; e < VEC; e += 4) *reinterpret_cast<float4*>(dst + e) = make_float4(acc[e], acc[e + 1], acc[e + 2], acc[e + 3]);
    if (threadIdx.x % LPR == 0) norm2[(long long)b * N + row] = n2;
  }
}

// grid = (ceil(N / (256 / (D/4))), B); D/4 lanes per token.
template <int D>
__global__ __launch_bounds__(256) void merge_similarity(const float* __restrict__ m, const float* __restrict__ norm2,
                                                        float* __restrict__ u, int32_t* __restrict__ blk, MergeGrid g,
                                                        int N) {
  constexpr int LPR = D / 4, RPW = 256 / LPR;
  const int b = blockIdx.y, i = blockIdx.x * RPW + threadIdx.x / LPR, c0 = (threadIdx.x % LPR) * 4;
  int j = 0, rank = 0;
  bool dst = false;
  float dot = 0.f;
  if (i < N) {
    const Tok c = coords(g, i);
    dst = is_dst(g, c);
    rank = dst_rank(g, c);  // c and its block's corner have the same quotients
    j = dst_index(g, c);
    const float4 a = *reinterpret_cast<const float4*>(m + ((long long)b * N + i) * D + c0);
    const float4 d = *reinterpret_cast<const float4*>(m + ((long long)b * N + j) * D + c0);
    dot = fmaf(a.x, d.x, fmaf(a.y, d.y, fmaf(a.z, d.z, a.w * d.w)));
  }
#pragma unroll
  for (int o = LPR / 2; o >= 1; o >>= 1) dot += __shfl_xor(dot, o);
  if (i < N && threadIdx.x % LPR == 0) {
    const float den = sqrtf(norm2[(long long)b * N + i]) * sqrtf(norm2[(long long)b * N + j]);
    u[(long long)b * N + i] = dst ? -INFINITY : (den > 0.f ? dot / den : 0.f);
    if (b == 0) blk[i] = rank | (dst ? (int)0x80000000 : 0);  // depends on the grid only
  }
}

// Order-preserving key of a canonicalised fp32: -0 == +0, NaN below everything.
__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t b = __float_as_uint(x);
  if ((b & 0x7fffffffu) > 0x7f800000u) return 0u;
  if (b == 0x80000000u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

// Exclusive prefixes of CH integers per thread in (chunk, thread) order: out[c] = everything in the
// chunks before c plus the threads before this one in chunk c; *carry_io carries the running total
// across calls (in: everything before chunk 0; out: plus these chunks).  `wave_tot` is LDS scratch of
// CH * kSelWaves + 1 ints.  Three barriers: wave scans, one wave scans the wave totals, read back.
template <int CH>
__device__ __forceinline__ void block_exclusive_chunks(int (&v)[CH], int* wave_tot, int* carry_io) {
  constexpr int ENTRIES = CH * kSelWaves, EPL = (ENTRIES + 63) / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc[CH];
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    inc[c] = v[c];
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(inc[c], o);
      if (lane >= o) inc[c] += t;
    }
    if (lane == 63) wave_tot[c * kSelWaves + wave] = inc[c];
  }
  __syncthreads();
  if (wave == 0) {  // exclusive scan of the ENTRIES wave totals, EPL consecutive entries per lane
    int x[EPL], sum = 0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const int id = lane * EPL + e;
      x[e] = id < ENTRIES ? wave_tot[id] : 0;
      sum += x[e];
    }
    int run = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(run, o);
      if (lane >= o) run += t;
    }
    if (lane == 63) wave_tot[ENTRIES] = run;  // grand total
    run -= sum;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const int id = lane * EPL + e;
      if (id < ENTRIES) wave_tot[id] = run;
      run += x[e];
    }
  }
  __syncthreads();
  const int carry = *carry_io;
#pragma unroll
  for (int c = 0; c < CH; ++c) v[c] = carry + wave_tot[c * kSelWaves + wave] + inc[c] - v[c];
  *carry_io = carry + wave_tot[ENTRIES];
  __syncthreads();
}

// Selection and row assignment, one workgroup per batch element (grid = B, 1024 threads).
// `blk[i]` = rank of token i's block among the destinations, bit 31 set at the destination itself
// (written by merge_similarity).  Tokens are handled in chunks of 4096: thread t owns the four
// consecutive tokens 4096 c + 4 t .. + 3 of chunk c, so loads and stores are 16 bytes per lane and
// contiguous across the wave, and (chunk, thread, e) order is raster order.
// Keys: 0 = not a source (destination or past the end), sources >= 1 (a NaN similarity, the lowest
// rank, maps to 1; every number maps above 0x007fffff).  The r-th largest key is found bit by bit
// from the top; r <= number of sources keeps the key-0 entries out of the result.
// CH > 0: all keys of up to 4096 * CH tokens stay in registers.  CH == 0: any N, keys are re-read
// from memory in every pass.
template <int CH>
__global__ __launch_bounds__(kSelThreads) void merge_select(const float* __restrict__ u, const int32_t* __restrict__ blk,
                                                            int32_t* __restrict__ row_of, int32_t* __restrict__ src_of,
                                                            int N, int n_dst, int r) {
  constexpr bool kReg = CH > 0;
  constexpr int C = kReg ? CH : 1;
  __shared__ int wave_cnt[2][kSelWaves];
  __shared__ int wave_tot[C * kSelWaves + 1];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* ub = u + (long long)b * N;
  int32_t* rob = row_of + (long long)b * N;
  int32_t* sob = src_of + (long long)b * (N - r);
  const int n_unmerged = N - n_dst - r;
  const int chunks = kReg ? CH : (N + 4 * kSelThreads - 1) / (4 * kSelThreads);
  const bool vec_ok = (N & 3) == 0;  // then every batch element's row of u, blk, row_of is 16-byte aligned

  auto load_keys = [&](int c, uint32_t (&key)[4], int (&bk)[4]) {
    const int i0 = (c * kSelThreads + tid) * 4;
    float x[4] = {0.f, 0.f, 0.f, 0.f};
    bk[0] = bk[1] = bk[2] = bk[3] = (int)0x80000000;
    if (vec_ok && i0 + 3 < N) {
      const float4 v = *reinterpret_cast<const float4*>(ub + i0);
      const int4 k4 = *reinterpret_cast<const int4*>(blk + i0);
      x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
      bk[0] = k4.x; bk[1] = k4.y; bk[2] = k4.z; bk[3] = k4.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (i0 + e < N) x[e] = ub[i0 + e], bk[e] = blk[i0 + e];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t k = order_key(x[e]);
      key[e] = (i0 + e < N && bk[e] >= 0) ? (k ? k : 1u) : 0u;
    }
  };

  uint32_t key[C][4];
  int bk[4];  // the partition words are only needed again at the very end: re-read there rather than kept
  if (kReg) {
#pragma unroll
    for (int c = 0; c < C; ++c) load_keys(c, key[c], bk);
  }

  // count of keys >= cand over the workgroup; `buf` alternates so that one barrier per call is enough
  auto count_ge = [&](uint32_t cand, int buf) {
    int n = 0;
    if (kReg) {
#pragma unroll
      for (int c = 0; c < C; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) n += key[c][e] >= cand ? 1 : 0;
    } else {
      for (int c = 0; c < chunks; ++c) {
        load_keys(c, key[0], bk);
#pragma unroll
        for (int e = 0; e < 4; ++e) n += key[0][e] >= cand ? 1 : 0;
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) n += __shfl_xor(n, o);
    if (lane == 0) wave_cnt[buf][wave] = n;
    __syncthreads();
    int all = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) all += wave_cnt[buf][w];
    return all;
  };

  uint32_t thr = 0xffffffffu;
  int need_eq = 0;
  if (r > 0) {  // uniform
    thr = 0u;
    int last_buf = 1;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = thr | (1u << bit);
      const int c = count_ge(cand, bit & 1);
      last_buf = bit & 1;
      if (c >= r) thr = cand;
      if (c == r) {  // uniform: exactly r keys are >= cand, they are the answer whatever the lower bits are
        thr = cand - 1u;
        break;
      }
    }
    // thr is the r-th largest key (or just below the r selected ones); thr + 1 counts the keys above it
    // (thr < 0xffffffff: no key is that large)
    need_eq = r - count_ge(thr + 1u, last_buf ^ 1);
    __syncthreads();
  }

  // ordered sweep.  Register version: all chunks at once (two scans in all); otherwise chunk by chunk.
  int eq_carry = 0, un_carry = 0;
  for (int c0 = 0; c0 < chunks; c0 += C) {  // one trip when kReg
    if (!kReg) load_keys(c0, key[0], bk);
    int rank[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
      rank[c] = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) rank[c] += key[c][e] == thr ? 1 : 0;
    }
    block_exclusive_chunks<C>(rank, wave_tot, &eq_carry);
    unsigned merged_bits[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
      int eq_rank = rank[c], un = 0;
      merged_bits[c] = 0u;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool eq = key[c][e] == thr;
        const bool merged = key[c][e] != 0u && (key[c][e] > thr || (eq && eq_rank < need_eq));
        eq_rank += eq ? 1 : 0;
        un += (key[c][e] != 0u && !merged) ? 1 : 0;
        merged_bits[c] |= merged ? 1u << e : 0u;
      }
      rank[c] = un;
    }
    block_exclusive_chunks<C>(rank, wave_tot, &un_carry);
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const int i0 = ((c0 + c) * kSelThreads + tid) * 4;
      if (i0 >= N) continue;
      if (kReg) {
        if (vec_ok && i0 + 3 < N) {
          const int4 k4 = *reinterpret_cast<const int4*>(blk + i0);
          bk[0] = k4.x; bk[1] = k4.y; bk[2] = k4.z; bk[3] = k4.w;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (i0 + e < N) bk[e] = blk[i0 + e];
        }
      }
      int un_rank = rank[c];
      int row[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool merged = (merged_bits[c] >> e) & 1u;
        // a destination's row, and the row a merged source reads back: the block's rank among the destinations
        row[e] = (key[c][e] == 0u || merged) ? n_unmerged + (bk[e] & 0x7fffffff) : un_rank++;
        if (i0 + e < N && !merged) sob[row[e]] = i0 + e;
      }
      if (vec_ok && i0 + 3 < N) {
        *reinterpret_cast<int4*>(rob + i0) = make_int4(row[0], row[1], row[2], row[3]);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (i0 + e < N) rob[i0 + e] = row[e];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// The same selection spread over the chip (used when the caller brings a workspace): a radix select
// over the 32-bit keys in three levels (8 + 12 + 12 bits), every level one launch of G = ceil(N / 2048)
// workgroups per batch element, then one launch that counts per slice and one that assigns the rows.
// Launches on one stream run one after the other, which is the only ordering used: no workgroup ever
// waits for another.  All counts are integers, so the atomic additions give the same result in any
// order, and ties are ranked by token index exactly as in the single-workgroup kernel.
//
// Workspace (int32) per batch element b:  state[8] = {D0, r1, D1, r2, thr, need_eq, -, -};
// hist1[4096], hist2[4096] (cleared by the first launch, filled by atomics); slice_hist0[G][256]
// (plain stores); slice_cnt[G][2] = {keys equal to thr, source keys below thr} of every slice.
constexpr int kRsThreads = 256, kRsPer = 8, kRsSlice = kRsThreads * kRsPer;
constexpr int kRsBins0 = 256, kRsBins = 4096, kRsState = 8;

struct RadixWs {
  int* state;        // [B][kRsState]
  int* hist1;        // [B][kRsBins]
  int* hist2;        // [B][kRsBins]
  int* slice_hist0;  // [B][G][kRsBins0]
  int* slice_cnt;    // [B][G][2]
};

// keys and partition words of the 8 consecutive tokens i0 .. i0 + 7 of batch element `ub`
__device__ __forceinline__ void rs_load(const float* __restrict__ ub, const int32_t* __restrict__ blk, int N, int i0,
                                        uint32_t (&key)[kRsPer], int (&bk)[kRsPer]) {
  float x[kRsPer];
#pragma unroll
  for (int e = 0; e < kRsPer; ++e) x[e] = 0.f, bk[e] = (int)0x80000000;
  if ((N & 3) == 0 && i0 + kRsPer - 1 < N) {  // rows of u and blk are 16-byte aligned
#pragma unroll
    for (int h = 0; h < kRsPer; h += 4) {
      const float4 v = *reinterpret_cast<const float4*>(ub + i0 + h);
      const int4 k4 = *reinterpret_cast<const int4*>(blk + i0 + h);
      x[h] = v.x; x[h + 1] = v.y; x[h + 2] = v.z; x[h + 3] = v.w;
      bk[h] = k4.x; bk[h + 1] = k4.y; bk[h + 2] = k4.z; bk[h + 3] = k4.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < kRsPer; ++e)
      if (i0 + e < N) x[e] = ub[i0 + e], bk[e] = blk[i0 + e];
  }
#pragma unroll
  for (int e = 0; e < kRsPer; ++e) {
    const uint32_t k = order_key(x[e]);
    key[e] = (i0 + e < N && bk[e] >= 0) ? (k ? k : 1u) : 0u;
  }
}

// Exclusive prefix of one int per thread over the 256 threads, and the total.  `lds` holds 4 ints.
__device__ __forceinline__ int rs_block_exclusive(int v, int* lds, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  __syncthreads();  // the previous use of lds is over
  if (lane == 63) lds[wave] = inc;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kRsThreads / 64; ++w) {
    before += w < wave ? lds[w] : 0;
    all += lds[w];
  }
  *total = all;
  return before + inc - v;
}

// The digit D that holds the r-th largest key of a level, given the level's counts h[0 .. BINS) in LDS
// (r >= 1 and at most the sum of the counts), and the rank that remains inside that digit:
// out[0] = D, out[1] = r - (keys with a larger digit).  Thread t owns BINS / 256 digits, highest first.
template <int BINS>
__device__ __forceinline__ void rs_pick(const int* h, int r, int* scan4, int* out) {
  constexpr int P = BINS / kRsThreads;
  const int top = BINS - 1 - (int)threadIdx.x * P;
  int own = 0;
#pragma unroll
  for (int p = 0; p < P; ++p) own += h[top - p];
  int total;
  int above = rs_block_exclusive(own, scan4, &total);
  if (threadIdx.x == 0) out[0] = 0, out[1] = 0;  // r == 0 or r beyond the total: no digit (callers do not use it then)
  __syncthreads();
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const int c = h[top - p];
    if (above < r && r <= above + c) out[0] = top - p, out[1] = r - above;
    above += c;
  }
  __syncthreads();
}

// 4096 counts of an earlier launch -> LDS, with all sixteen loads of a thread in flight together
__device__ __forceinline__ void rs_fetch_counts(const int* __restrict__ src, int* h) {
  int t[kRsBins / kRsThreads];
#pragma unroll
  for (int k = 0; k < kRsBins / kRsThreads; ++k) t[k] = src[k * kRsThreads + threadIdx.x];
#pragma unroll
  for (int k = 0; k < kRsBins / kRsThreads; ++k) h[k * kRsThreads + threadIdx.x] = t[k];
}

// level 0: counts of the top 8 key bits of this slice; the first slice also clears the level-1/2 counts
__global__ __launch_bounds__(kRsThreads) void rs_hist0(const float* __restrict__ u, const int32_t* __restrict__ blk, int N,
                                                       RadixWs ws) {
  __shared__ int h[kRsBins0];
  const int b = blockIdx.y, g = blockIdx.x, G = gridDim.x, tid = threadIdx.x;
  h[tid] = 0;
  __syncthreads();
  uint32_t key[kRsPer];
  int bk[kRsPer];
  rs_load(u + (long long)b * N, blk, N, g * kRsSlice + tid * kRsPer, key, bk);
#pragma unroll
  for (int e = 0; e < kRsPer; ++e)
    if (key[e]) atomicAdd(&h[key[e] >> 24], 1);
  __syncthreads();
  ws.slice_hist0[((long long)b * G + g) * kRsBins0 + tid] = h[tid];
  if (g == 0) {
    for (int i = tid; i < kRsBins; i += kRsThreads) ws.hist1[(long long)b * kRsBins + i] = 0, ws.hist2[(long long)b * kRsBins + i] = 0;
  }
}

// levels 1 and 2: pick the digit of the level above from its counts, then count this level's 12 bits over the keys
// that carry the digits picked so far
template <int LEVEL>
__global__ __launch_bounds__(kRsThreads) void rs_hist12(const float* __restrict__ u, const int32_t* __restrict__ blk, int N,
                                                        int r, RadixWs ws) {
  __shared__ int h[kRsBins];
  __shared__ int scan4[4], out[2];
  const int b = blockIdx.y, g = blockIdx.x, G = gridDim.x, tid = threadIdx.x;
  int* state = ws.state + (long long)b * kRsState;
  // every global read this workgroup needs is requested up front (the words of the earlier launches come from
  // another XCD's writes, i.e. from memory: a couple of microseconds each if they were taken one after the other)
  const int st0 = LEVEL == 2 ? state[0] : 0, st1 = LEVEL == 2 ? state[1] : 0;
  uint32_t key[kRsPer];
  int bk[kRsPer];
  rs_load(u + (long long)b * N, blk, N, g * kRsSlice + tid * kRsPer, key, bk);
  uint32_t prefix;  // the key bits above this level's 12
  if constexpr (LEVEL == 1) {
    int s = 0;
#pragma unroll 8
    for (int gg = 0; gg < G; ++gg) s += ws.slice_hist0[((long long)b * G + gg) * kRsBins0 + tid];
    h[tid] = s;
    __syncthreads();
    rs_pick<kRsBins0>(h, r, scan4, out);
    if (g == 0 && tid == 0) state[0] = out[0], state[1] = out[1];
    prefix = (uint32_t)out[0];
  } else {
    rs_fetch_counts(ws.hist1 + (long long)b * kRsBins, h);
    __syncthreads();
    rs_pick<kRsBins>(h, st1, scan4, out);
    if (g == 0 && tid == 0) state[2] = out[0], state[3] = out[1];
    prefix = ((uint32_t)st0 << 12) | (uint32_t)out[0];
  }
  __syncthreads();  // everyone has read h and out
  for (int i = tid; i < kRsBins; i += kRsThreads) h[i] = 0;
  __syncthreads();
  constexpr int SHIFT = LEVEL == 1 ? 12 : 0;
#pragma unroll
  for (int e = 0; e < kRsPer; ++e)
    if (key[e] && (key[e] >> (SHIFT + 12)) == prefix) atomicAdd(&h[(key[e] >> SHIFT) & (kRsBins - 1)], 1);
  __syncthreads();
  int* dst = (LEVEL == 1 ? ws.hist1 : ws.hist2) + (long long)b * kRsBins;
  for (int i = tid; i < kRsBins; i += kRsThreads)
    if (h[i]) atomicAdd(&dst[i], h[i]);
}

// the threshold key and the number of ties to take, then this slice's counts against it
__global__ __launch_bounds__(kRsThreads) void rs_count(const float* __restrict__ u, const int32_t* __restrict__ blk, int N,
                                                       int r, RadixWs ws) {
  __shared__ int h[kRsBins];
  __shared__ int scan4[4], out[2];
  const int b = blockIdx.y, g = blockIdx.x, G = gridDim.x, tid = threadIdx.x;
  int* state = ws.state + (long long)b * kRsState;
  const int st0 = state[0], st2 = state[2], st3 = state[3];  // (unused garbage when r == 0)
  uint32_t key[kRsPer];
  int bk[kRsPer];
  rs_load(u + (long long)b * N, blk, N, g * kRsSlice + tid * kRsPer, key, bk);
  uint32_t thr = 0xffffffffu;  // r == 0: nothing is merged (no key is that large)
  int need_eq = 0;
  if (r > 0) {
    rs_fetch_counts(ws.hist2 + (long long)b * kRsBins, h);
    __syncthreads();
    rs_pick<kRsBins>(h, st3, scan4, out);
    thr = ((uint32_t)st0 << 24) | ((uint32_t)st2 << 12) | (uint32_t)out[0];
    need_eq = out[1];
  }
  if (g == 0 && tid == 0) state[4] = (int)thr, state[5] = need_eq;
  int eq = 0, lt = 0;
#pragma unroll
  for (int e = 0; e < kRsPer; ++e) {
    eq += key[e] == thr ? 1 : 0;
    lt += (key[e] != 0u && key[e] < thr) ? 1 : 0;
  }
  int eq_all, lt_all;
  rs_block_exclusive(eq, scan4, &eq_all);
  rs_block_exclusive(lt, scan4, &lt_all);
  if (tid == 0) {
    ws.slice_cnt[((long long)b * G + g) * 2] = eq_all;
    ws.slice_cnt[((long long)b * G + g) * 2 + 1] = lt_all;
  }
}

// rows of the merged sequence: the ordered sweep of the single-workgroup kernel, one slice per workgroup, with the
// counts of the slices before it as its carry
__global__ __launch_bounds__(kRsThreads) void rs_assign(const float* __restrict__ u, const int32_t* __restrict__ blk,
                                                        int32_t* __restrict__ row_of, int32_t* __restrict__ src_of, int N,
                                                        int n_dst, int r, RadixWs ws) {
  __shared__ int scan4[4];
  const int b = blockIdx.y, g = blockIdx.x, G = gridDim.x, tid = threadIdx.x;
  const int* state = ws.state + (long long)b * kRsState;
  const uint32_t thr = (uint32_t)state[4];
  const int need_eq = state[5];
  const int i0 = g * kRsSlice + tid * kRsPer;
  uint32_t key[kRsPer];
  int bk[kRsPer];
  rs_load(u + (long long)b * N, blk, N, i0, key, bk);
  const int n_unmerged = N - n_dst - r;
  int32_t* rob = row_of + (long long)b * N;
  int32_t* sob = src_of + (long long)b * (N - r);
  // ties and lower keys in the slices before this one
  int eq_b = 0, lt_b = 0;
  for (int gg = tid; gg < g; gg += kRsThreads) {
    eq_b += ws.slice_cnt[((long long)b * G + gg) * 2];
    lt_b += ws.slice_cnt[((long long)b * G + gg) * 2 + 1];
  }
  int eq_before, lt_before;
  rs_block_exclusive(eq_b, scan4, &eq_before);
  rs_block_exclusive(lt_b, scan4, &lt_before);
  const int un_before = lt_before + max(0, eq_before - need_eq);  // ties beyond the first need_eq stay unmerged

  int eq = 0;
#pragma unroll
  for (int e = 0; e < kRsPer; ++e) eq += key[e] == thr ? 1 : 0;
  int unused;
  int eq_rank = eq_before + rs_block_exclusive(eq, scan4, &unused);
  unsigned merged_bits = 0u;
  int un = 0;
#pragma unroll
  for (int e = 0; e < kRsPer; ++e) {
    const bool is_eq = key[e] == thr;
    const bool merged = key[e] != 0u && (key[e] > thr || (is_eq && eq_rank < need_eq));
    eq_rank += is_eq ? 1 : 0;
    un += (key[e] != 0u && !merged) ? 1 : 0;
    merged_bits |= merged ? 1u << e : 0u;
  }
  int un_rank = un_before + rs_block_exclusive(un, scan4, &unused);
  if (i0 >= N) return;
  int row[kRsPer];
#pragma unroll
  for (int e = 0; e < kRsPer; ++e) {
    const bool merged = (merged_bits >> e) & 1u;
    // a destination's row, and the row a merged source reads back: the block's rank among the destinations
    row[e] = (key[e] == 0u || merged) ? n_unmerged + (bk[e] & 0x7fffffff) : un_rank++;
    // (the bound holds by construction; it keeps a partition array that does not belong to this grid from writing past src_of)
    if (i0 + e < N && !merged && (unsigned)row[e] < (unsigned)(N - r)) sob[row[e]] = i0 + e;
  }
  if ((N & 3) == 0 && i0 + kRsPer - 1 < N) {
    *reinterpret_cast<int4*>(rob + i0) = make_int4(row[0], row[1], row[2], row[3]);
    *reinterpret_cast<int4*>(rob + i0 + 4) = make_int4(row[4], row[5], row[6], row[7]);
  } else {
#pragma unroll
    for (int e = 0; e < kRsPer; ++e)
      if (i0 + e < N) rob[i0 + e] = row[e];
  }
}

// grid = (dst_wgs + copy_wgs, Hh, B).  Nm = N - r valid merged rows, of which the last nT * nH * nW are the
// destinations in ascending raster order and the others copies of token src_of[p]; rows Nm <= p < Np are padding.
// A group of D / VEC lanes owns a row piece by piece (16 bytes per lane, kept as raw chunks while in flight).
// The first dst_wgs workgroups take the destination and padding rows, one per lane group: they cost several dependent
// reads each, so they start first.  The others copy CR rows per lane group, all their loads in flight together.
template <typename T, int D, int CR>
__global__ __launch_bounds__(256) void merge_rows(const T* __restrict__ x, const int32_t* __restrict__ row_of,
                                                  const int32_t* __restrict__ src_of, T* __restrict__ out, MergeGrid g,
                                                  int N, int Nm, int Np, int Hh, int dst_wgs) {
  constexpr int VEC = Row<T>::kElems, LPR = D / VEC, RPW = 256 / LPR;
  const int b = blockIdx.z, h = blockIdx.y, lg = threadIdx.x / LPR, c0 = (threadIdx.x % LPR) * VEC;
  const int n_unmerged = Nm - g.nT * g.nH * g.nW;
  const T* xb = x + ((long long)(b * Hh + h) * N) * D + c0;
  T* ob = out + ((long long)(b * Hh + h) * Np) * D + c0;
  if ((int)blockIdx.x >= dst_wgs) {  // copies, byte for byte
    const int p0 = ((int)blockIdx.x - dst_wgs) * (RPW * CR) + lg;
    int src[CR];
#pragma unroll
    for (int k = 0; k < CR; ++k)  // (device contents are not trusted with addresses: the token index is clamped into the grid)
      src[k] = min(max(src_of[(long long)b * Nm + min(p0 + k * RPW, n_unmerged - 1)], 0), N - 1);
    chunk_t raw[CR];
#pragma unroll
    for (int k = 0; k < CR; ++k) raw[k] = __builtin_nontemporal_load(reinterpret_cast<const chunk_t*>(xb + (long long)src[k] * D));
#pragma unroll
    for (int k = 0; k < CR; ++k)
      if (p0 + k * RPW < n_unmerged) *reinterpret_cast<chunk_t*>(ob + (long long)(p0 + k * RPW) * D) = raw[k];
    return;
  }
  const int p = n_unmerged + (int)blockIdx.x * RPW + lg;
  if (p >= Np) return;
  ob += (long long)p * D;
  if (p >= Nm) {  // padding rows are written as zero
    *reinterpret_cast<chunk_t*>(ob) = chunk_t{0u, 0u, 0u, 0u};
    return;
  }
  // the destination's coordinates follow from the row number alone: no look-up waits for src_of
  const int rank = p - n_unmerged, bt = rank / (g.nH * g.nW), rem = rank - bt * g.nH * g.nW, bh = rem / g.nW;
  Tok c;
  c.t = bt * g.st;
  c.h = bh * g.sh;
  c.w = (rem - bh * g.nW) * g.sw;
  const int s = (c.t * g.H + c.h) * g.W + c.w;
  // A destination: the mean of itself and the tokens of its block that read back from row p.  2x2x2 blocks (the usual
  // case) have all seven look-ups in flight together, then eight row pieces without a branch between them: a slot
  // that does not take part re-reads the destination's own piece (the same cache line) and is left out of the sum.
  const int32_t* ro = row_of + (long long)b * N;
  const int et = min(g.st, g.T - c.t), eh = min(g.sh, g.H - c.h), ew = min(g.sw, g.W - c.w);
  float acc[VEC];
  int count = 1;
  if (g.st == 2 && g.sh == 2 && g.sw == 2) {
    int kk[8], rk[8];
    kk[0] = s;
#pragma unroll
    for (int q = 1; q < 8; ++q) {
      const int lw = q & 1, lh = (q >> 1) & 1, lt = q >> 2;
      const bool inside = lt < et && lh < eh && lw < ew;
      kk[q] = inside ? ((c.t + lt) * g.H + c.h + lh) * g.W + c.w + lw : s;
      rk[q] = ro[kk[q]];  // (the destination's own word is p as well: `inside` keeps it out)
      rk[q] = inside ? rk[q] : -1;
    }
    bool use[8];
#pragma unroll
    for (int q = 1; q < 8; ++q) {
      use[q] = rk[q] == p;
      kk[q] = use[q] ? kk[q] : s;
    }
    chunk_t raw[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) raw[q] = *reinterpret_cast<const chunk_t*>(xb + (long long)kk[q] * D);
    widen<T>(raw[0], acc);
#pragma unroll
    for (int q = 1; q < 8; ++q) {  // same order of additions as the general walk below
      float v[VEC];
      widen<T>(raw[q], v);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] = use[q] ? acc[e] + v[e] : acc[e];
      count += use[q] ? 1 : 0;
    }
  } else {  // any other block shape: walk the block
    Row<T>::load(xb + (long long)s * D, acc);
    for (int lt = 0; lt < et; ++lt)
      for (int lh = 0; lh < eh; ++lh)
        for (int lw = 0; lw < ew; ++lw) {
          const int k = ((c.t + lt) * g.H + c.h + lh) * g.W + c.w + lw;
          if (k != s && ro[k] == p) {
            float v[VEC];
            Row<T>::load(xb + (long long)k * D, v);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += v[e];
            ++count;
          }
        }
  }
  if (count > 1) {
    const float inv = 1.0f / (float)count;
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] *= inv;
  }
  Row<T>::store(ob, acc);
}


// grid = (ceil(N / 64), B*Hh): 64 raster tokens per workgroup, <= 4 pieces of 16 bytes per lane.
template <int CHUNKS>
__global__ __launch_bounds__(CHUNKS >= 32 ? 512 : 256) void unmerge_rows(const unsigned char* __restrict__ y,
                                                                         const int32_t* __restrict__ row_of,
                                                                         unsigned char* __restrict__ out, int N, int Np,
                                                                         int Hh) {
  constexpr int kThreads = CHUNKS >= 32 ? 512 : 256;
  constexpr int kRowBytes = CHUNKS * 16, PER_THREAD = kBlock * CHUNKS / kThreads;
  __shared__ int row[kBlock];
  const int tid = threadIdx.x, k0 = blockIdx.x * kBlock, bh = blockIdx.y, b = bh / Hh;
  if (tid < kBlock) row[tid] = k0 + tid < N ? min(max(row_of[(long long)b * N + k0 + tid], 0), Np - 1) : 0;  // clamped into y
  __syncthreads();
  const unsigned char* src = y + (long long)bh * Np * kRowBytes;
  unsigned char* dst = out + ((long long)bh * N + k0) * kRowBytes;
  chunk_t val[PER_THREAD];
#pragma unroll
  for (int it = 0; it < PER_THREAD; ++it) {
    const int c = it * kThreads + tid, rr = c / CHUNKS, ch = c - rr * CHUNKS;
    val[it] = chunk_t{0u, 0u, 0u, 0u};
    if (k0 + rr < N) val[it] = *reinterpret_cast<const chunk_t*>(src + (long long)row[rr] * kRowBytes + ch * 16);
  }
#pragma unroll
  for (int it = 0; it < PER_THREAD; ++it) {
    const int c = it * kThreads + tid, rr = c / CHUNKS, ch = c - rr * CHUNKS;
    if (k0 + rr < N) *reinterpret_cast<chunk_t*>(dst + (long long)rr * kRowBytes + ch * 16) = val[it];
  }
}

}  // namespace

// ws: m [B, N, d] fp32, then |m|^2 [B, N] fp32
hipError_t launch_merge_similarity(const void* k, const Dims& s, const MergeGrid& g, int N, float* u, int32_t* blk,
                                   float* ws, hipStream_t st) {
  float* m = ws;
  float* n2 = ws + (long long)s.B * N * s.d;
  const int vec = s.bf16 ? 8 : 4, rpw = 256 / (s.d / vec);
  const dim3 grid_d((unsigned)((N + rpw - 1) / rpw), (unsigned)s.B);
  if (s.bf16) {
    if (s.d == 128) merge_descriptors<uint16_t, 128><<<grid_d, 256, 0, st>>>(static_cast<const uint16_t*>(k), m, n2, N, s.Hh);
    else merge_descriptors<uint16_t, 64><<<grid_d, 256, 0, st>>>(static_cast<const uint16_t*>(k), m, n2, N, s.Hh);
  } else {
    if (s.d == 128) merge_descriptors<float, 128><<<grid_d, 256, 0, st>>>(static_cast<const float*>(k), m, n2, N, s.Hh);
    else merge_descriptors<float, 64><<<grid_d, 256, 0, st>>>(static_cast<const float*>(k), m, n2, N, s.Hh);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int rpw2 = 256 / (s.d / 4);
  const dim3 grid_s((unsigned)((N + rpw2 - 1) / rpw2), (unsigned)s.B);
  if (s.d == 128) merge_similarity<128><<<grid_s, 256, 0, st>>>(m, n2, u, blk, g, N);
  else merge_similarity<64><<<grid_s, 256, 0, st>>>(m, n2, u, blk, g, N);
  return hipGetLastError();
}

size_t merge_plan_workspace_bytes(int B, int N) {
  const size_t G = (size_t)(N + kRsSlice - 1) / kRsSlice;
  return (size_t)B * (kRsState + 2 * kRsBins + G * (kRsBins0 + 2)) * sizeof(int);
}

hipError_t launch_merge_select(const float* u, const int32_t* blk, const MergeGrid& g, int B, int N, int r, int32_t* row_of,
                               int32_t* src_of, void* ws, hipStream_t st) {
  const int n_dst = g.nT * g.nH * g.nW;
  if (ws) {
    const unsigned G = (unsigned)((N + kRsSlice - 1) / kRsSlice);
    RadixWs w;
    w.state = static_cast<int*>(ws);
    w.hist1 = w.state + (size_t)B * kRsState;
    w.hist2 = w.hist1 + (size_t)B * kRsBins;
    w.slice_hist0 = w.hist2 + (size_t)B * kRsBins;
    w.slice_cnt = w.slice_hist0 + (size_t)B * G * kRsBins0;
    const dim3 grid(G, (unsigned)B);
    if (r > 0) {
      rs_hist0<<<grid, kRsThreads, 0, st>>>(u, blk, N, w);
      rs_hist12<1><<<grid, kRsThreads, 0, st>>>(u, blk, N, r, w);
      rs_hist12<2><<<grid, kRsThreads, 0, st>>>(u, blk, N, r, w);
    }
    rs_count<<<grid, kRsThreads, 0, st>>>(u, blk, N, r, w);
    rs_assign<<<grid, kRsThreads, 0, st>>>(u, blk, row_of, src_of, N, n_dst, r, w);
    return hipGetLastError();
  }
  if (N <= kSelThreads * 4 * 8)
    merge_select<8><<<(unsigned)B, kSelThreads, 0, st>>>(u, blk, row_of, src_of, N, n_dst, r);
  else if (N <= kSelThreads * 4 * 20)
    merge_select<20><<<(unsigned)B, kSelThreads, 0, st>>>(u, blk, row_of, src_of, N, n_dst, r);
  else
    merge_select<0><<<(unsigned)B, kSelThreads, 0, st>>>(u, blk, row_of, src_of, N, n_dst, r);
  return hipGetLastError();
}

hipError_t launch_merge_rows(const void* x, const Dims& s, const MergeGrid& g, int N, const int32_t* row_of,
                             const int32_t* src_of, void* out, hipStream_t st) {
  const int vec = s.bf16 ? 8 : 4, rpw = 256 / (s.d / vec);
  constexpr int CR = USV_MERGE_COPY_ROWS;
  const int n_unmerged = s.Nv - g.nT * g.nH * g.nW;
  const int dst_wgs = (s.N - n_unmerged + rpw - 1) / rpw, copy_wgs = (n_unmerged + rpw * CR - 1) / (rpw * CR);
  const dim3 grid((unsigned)(dst_wgs + copy_wgs), (unsigned)s.Hh, (unsigned)s.B);
#define USV_MERGE_ROWS(T, DD)                                                                                               \
  merge_rows<T, DD, CR><<<grid, 256, 0, st>>>(static_cast<const T*>(x), row_of, src_of, static_cast<T*>(out), g, N, s.Nv, s.N, \
                                              s.Hh, dst_wgs)
  if (s.bf16) {
    if (s.d == 128) USV_MERGE_ROWS(uint16_t, 128);
    else USV_MERGE_ROWS(uint16_t, 64);
  } else {
    if (s.d == 128) USV_MERGE_ROWS(float, 128);
    else USV_MERGE_ROWS(float, 64);
  }
#undef USV_MERGE_ROWS
  return hipGetLastError();
}

hipError_t launch_unmerge_rows(const void* y, const Dims& s, int N, const int32_t* row_of, void* out, hipStream_t st) {
  const int chunks = s.d * (s.bf16 ? 2 : 4) / 16;
  const dim3 grid((unsigned)((N + kBlock - 1) / kBlock), (unsigned)s.bh());
  auto Y = static_cast<const unsigned char*>(y);
  auto O = static_cast<unsigned char*>(out);
  if (chunks == 8) unmerge_rows<8><<<grid, 256, 0, st>>>(Y, row_of, O, N, s.N, s.Hh);
  else if (chunks == 16) unmerge_rows<16><<<grid, 256, 0, st>>>(Y, row_of, O, N, s.N, s.Hh);
  else if (chunks == 32) unmerge_rows<32><<<grid, 512, 0, st>>>(Y, row_of, O, N, s.N, s.Hh);
  else return hipErrorInvalidValue;  // unreachable: d in {64, 128}, bf16 or fp32
  return hipGetLastError();
}

}  // namespace usv
