// Stage 3, bf16 path: block-sparse flash attention on the gfx950 matrix cores
// (masked-attention equation, paper Section 3.2; only listed K/V cubes are touched).
//
// Work decomposition (one workgroup = 4 wavefronts = one 64-row query block):
//   wave (qh, kh): query rows 32*qh .. +32, keys 32*kh .. +32 of every listed 64-key tile.
//   Each wave runs an independent online softmax over its half of the keys; the two key halves
//   are merged once, at the end, through LDS.  All four waves share the K/V tile in LDS, so a
//   tile is fetched from L2/HBM once per query block.
//
// Matrix-core mapping (v_mfma_f32_16x16x32_bf16, fp32 accumulate; lane = (c, G) with c = lane % 16,
// G = lane / 16; the A operand holds row c, contraction slots 8 G .. 8 G + 7, the B operand column c
// and the same slots, the result column c, rows 4 G .. 4 G + 3):
//   S^T (16 keys x 16 queries) = K_tile (A, rows = keys) x Q^T (B, cols = queries), 4 steps over d = 128
//   O^T (16 d    x 16 queries) = V^T    (A, rows = d)    x P^T (B, cols = queries), ONE step over 32 keys
// A wave's 32 keys x 32 queries are 2 x 2 such tiles.  Working on the transposes keeps a query in a
// lane column: lane (c, G) holds queries c and 16 + c, eight keys of each (16 mt + 4 G + r), and those
// eight S^T accumulator values are, as they stand, the eight contraction slots of the P^T operand for
// that query (the contraction index of an MFMA can be enumerated in any order as long as both operands
// agree, so V^T is read in the order the accumulators hold the keys).  Row statistics therefore stay
// in the lane; only a raise of the reference maximum (rare) looks across the four lanes of a query.
// V^T fragments come from the row-major V tile with the LDS transpose read ds_read_b64_tr_b16.
// The 16x16x32 shape was chosen over 32x32x16 by measurement: the same flops draw less power, and
// under this kernel the chip runs at its power limit, where less energy per tile is more clock.
//
// What bounds the kernel, measured on MI355X: a wavefront issues at most one instruction (of any
// kind) every ~8 clocks, a tile's 32 MFMAs per wave occupy the matrix pipe for 512 clocks, and the
// CU's vector-memory path moves 64 B/clk (a 64x64 tile needs 32 KiB of K and V: 512 clocks as
// well).  With two workgroups per CU the chip then sits at its power limit
// (it clocks this kernel at ~1.7 GHz of 2.4) and, for lists without locality, near what the
// L2-miss path delivers (~7 TB/s), so every instruction and every byte moved costs clock.
// The design goal is therefore few instructions per tile and two or three
// workgroups per CU (waves per SIMD) that cover each other's issue gaps and waits:
//   - K/V tiles go global -> LDS directly (global_load_lds, 16 bytes per lane, no register
//     staging, M0 set once per tile) through a ring of tile slots K(n), V(n), K(n+1), ... (3 as launched);
//     a slot is refilled as soon as the barrier after its last reader has passed;
//   - the 16-byte chunks of a row are XOR-permuted on the way in (applied to the global address;
//     the LDS side of the DMA is lane-linear) so that both the 16-byte K fragment reads and the
//     transposing V reads are bank-conflict free;
//   - softmax in the log2 domain; the running max is only raised when a row's tile max exceeds it
//     by more than kRescaleSlack, so the O rescale is skipped on almost every tile.
#include <type_traits>

#include "usv_internal.h"

namespace usv {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4v;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short short8v;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// Accumulators are kept four 16x16 tiles to a 16-register tuple and the MFMAs work on quarter q of it:
// with one allocation unit per tuple the compiler updates the accumulators in place (given 64 separate
// 4-register values it rotated them through fresh registers and copied all of them back on every tile).
__device__ __forceinline__ f32x4 quarter(const f32x16& v, int q) {
  switch (q) {
    case 0: return __builtin_shufflevector(v, v, 0, 1, 2, 3);
    case 1: return __builtin_shufflevector(v, v, 4, 5, 6, 7);
    case 2: return __builtin_shufflevector(v, v, 8, 9, 10, 11);
    default: return __builtin_shufflevector(v, v, 12, 13, 14, 15);
  }
}
__device__ __forceinline__ void set_quarter(f32x16& v, int q, const f32x4& c) {
  const f32x16 w = __builtin_shufflevector(c, c, 0, 1, 2, 3, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1);
  switch (q) {
    case 0: v = __builtin_shufflevector(v, w, 16, 17, 18, 19, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15); break;
    case 1: v = __builtin_shufflevector(v, w, 0, 1, 2, 3, 16, 17, 18, 19, 8, 9, 10, 11, 12, 13, 14, 15); break;
    case 2: v = __builtin_shufflevector(v, w, 0, 1, 2, 3, 4, 5, 6, 7, 16, 17, 18, 19, 12, 13, 14, 15); break;
    default: v = __builtin_shufflevector(v, w, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 16, 17, 18, 19); break;
  }
}

constexpr int kThreads = 256;
constexpr float kRescaleSlack = 8.0f;  // log2 units
// The probabilities are computed as 2^(logit - m - p_shift): the common factor 2^-p_shift cancels in
// sum(p v) / sum(p), and it pushes every p below tau = 2^-(126 - p_shift) of the row's reference under
// the fp32 normal range, where v_exp_f32 returns an exact 0.  Zero operands keep the matrix cores'
// multipliers quiet, which matters because the chip is power-limited under this kernel (measured:
// +3 % at tau = 2^-24, +10 % on dense lists at tau = 2^-16).  The dropped mass of a row is below
// keys * tau of its largest term; the launcher picks tau so that this is at most 2^-12 (2.4e-4
// relative, against an error budget of ~2.5e-3), i.e. tau = 2^-12 / (keys of the longest list).
constexpr int kDropLog2 = 12;

template <int D>
struct Tile {
  static constexpr int kChunks = D / 8;           // 16-byte chunks per row
  static constexpr int kRowBytes = D * 2;
  static constexpr int kBytes = kBlock * D * 2;   // one K or V tile
  static constexpr int kDmaPerWave = kBytes / 1024 / 4;  // 1 KiB DMA instructions per wave per tile
  static constexpr int kRowsPerDma = 1024 / kRowBytes;
  // K: lanes 0..15 of a fragment read hit 16 consecutive rows at one chunk column.
  __device__ static int k_swz(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
  // V: a transposing read addresses, per 16-lane group, 4 consecutive rows x 32 bytes (2 chunks) and
  // one LDS cycle serves two groups, i.e. 8 consecutive rows at the same pair of chunks; XOR-ing the
  // chunk-pair index with the row spreads those 8 rows over all banks.  Rows r and r + 16 share the
  // permutation, so the two reads of a fragment differ by a constant.
  __device__ static int v_swz(int row) { return D == 128 ? ((row & 7) << 1) : (((row >> 1) & 3) << 1); }
  __device__ static int k_off(int row, int chunk) { return row * kRowBytes + ((chunk ^ k_swz(row)) << 4); }
  __device__ static int v_off(int row, int chunk) { return row * kRowBytes + ((chunk ^ v_swz(row)) << 4); }
};

__device__ __forceinline__ float4 load_bf16x4(const uint16_t* p) {
  // (the gates of the fused second branch: read once, so a streaming read)
  typedef __attribute__((__vector_size__(2 * sizeof(unsigned)))) unsigned u32x2;
  const u32x2 ww = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
  const uint2 w = make_uint2(ww[0], ww[1]);
  return make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                     __uint_as_float(w.y & 0xffff0000u));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// v_permlane32_swap on two copies of x leaves (x of lane l % 32, x of lane l % 32 + 32) in both lanes:
// one VALU op, no LDS round trip.
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  lo = __uint_as_float(r[0]);
  hi = __uint_as_float(r[1]);
}

// Max of the 8 accumulator values a lane holds for one query, in 4 instructions.  One assembly block:
// v_max3 without the NaN-quieting moves the compiler adds around fmaxf (the inputs are never NaN).
__device__ __forceinline__ float max8(float a0, float a1, float a2, float a3, float b0, float b1, float b2, float b3) {
  float x, y;
  asm("v_max3_f32 %0, %2, %3, %4\n\t"
      "v_max3_f32 %1, %5, %6, %7\n\t"
      "v_max3_f32 %0, %0, %8, %9\n\t"
      "v_max_f32 %0, %0, %1"
      : "=&v"(x), "=&v"(y)
      : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(b0), "v"(b1), "v"(b2), "v"(b3));
  return x;
}

// The four lanes c, c + 16, c + 32, c + 48 hold the keys of one query.  v_permlane16_swap on two copies
// of x leaves (x of the even 16-lane row, x of the odd row) of each row pair in both rows, and
// v_permlane32_swap does the same for the two wave halves: two VALU ops per step, no LDS round trip.
__device__ __forceinline__ void row_pair(float x, float& even, float& odd) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  even = __uint_as_float(r[0]);
  odd = __uint_as_float(r[1]);
}
__device__ __forceinline__ float max_over_groups(float x) {
  float a, b;
  row_pair(x, a, b);
  x = fmaxf(a, b);
  both_halves(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float sum_over_groups(float x) {
  float a, b;
  row_pair(x, a, b);
  x = a + b;
  both_halves(x, a, b);
  return a + b;
}

__device__ __forceinline__ unsigned lds_address(const void* p) {  // LDS byte address of a __shared__ pointer
  return (unsigned)(uintptr_t)p;
}

// One wave's share of a tile, global -> LDS: N instructions of 16 bytes per lane.  Instruction `it`
// reads gbase + voff[it] + 1024*it per lane and lands at lds_addr + 1024*it + 16*lane (the
// instruction offset applies to both addresses).  Inline assembly so that the compiler does not
// pair the DMA with a conservative "wait for all memory" before the next LDS read of ANOTHER slot;
// completion is awaited explicitly (vmcnt) where the pipeline needs it.  M0 carries the LDS
// address; nothing else in this kernel uses M0 (no LDS-direct reads, no relative register indexing: every
// register array is indexed by compile-time constants), and the compiler refuses M0 on a clobber list (reserved
// register), so every block writes M0 itself right before the instructions that read it.
template <int N>
__device__ __forceinline__ void dma_tile(const void* gbase, const int (&voff)[N], unsigned lds_addr);
template <>
__device__ __forceinline__ void dma_tile<4>(const void* gbase, const int (&voff)[4], unsigned lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "global_load_lds_dwordx4 %1, %5\n\t"
      "global_load_lds_dwordx4 %2, %5 offset:1024\n\t"
      "global_load_lds_dwordx4 %3, %5 offset:2048\n\t"
      "global_load_lds_dwordx4 %4, %5 offset:3072"
      :
      : "s"(lds_addr), "v"(voff[0]), "v"(voff[1]), "v"(voff[2]), "v"(voff[3]), "s"(gbase)
      : "memory");
}
template <>
__device__ __forceinline__ void dma_tile<2>(const void* gbase, const int (&voff)[2], unsigned lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "global_load_lds_dwordx4 %1, %3\n\t"
      "global_load_lds_dwordx4 %2, %3 offset:1024"
      :
      : "s"(lds_addr), "v"(voff[0]), "v"(voff[1]), "s"(gbase)
      : "memory");
}

// SLOTS (odd) = tile slots of the LDS ring; a tile is requested LEAD = (SLOTS-1)/2 tiles before it
// is used.  WGS = workgroups (= waves per SIMD) the register and LDS budget is sized for.
// RASTER: Q, K, V and the output are in raster token order (any strides); `ras.order[p]` gives the
// raster index of cube-major position p.  Every wave fetches the 16 order entries of the rows it
// requests ahead of the tile (one more 4-byte-per-lane DMA per tile, into a small LDS ring that only
// this wave reads), turns them into the per-lane global offsets of its DMA instructions, and the
// epilogue stores each row at its raster position: no reordered copy of any tensor exists.
template <int D, bool OUT_F32, int SLOTS, int WGS, bool RASTER>
__global__ __launch_bounds__(kThreads, WGS) void attn_bf16(const uint16_t* __restrict__ q,
                                                                const uint16_t* __restrict__ k,
                                                                const uint16_t* __restrict__ v,
                                                                const int32_t* __restrict__ idx,
                                                                const int32_t* __restrict__ cnt,
                                                                void* __restrict__ out, float* __restrict__ lse,
                                                                int nb, int Nv, int kmax, float scale_log2e,
                                                                float p_shift, int total, int per_xcd, FuseArgs fuse,
                                                                RasterArgs ras, const int32_t* __restrict__ work_order,
                                                                int stream_out) {
  using T = Tile<D>;
  constexpr int KS = D / 32;  // MFMA k-steps of the QK^T product
  constexpr int DT = D / 16;  // 16-wide d sub-tiles of the output
  constexpr int kDma = T::kDmaPerWave;
  constexpr int kSlots = SLOTS;
  constexpr int LEAD = (SLOTS - 1) / 2;
  static_assert(SLOTS % 2 == 1 && SLOTS >= 3, "odd ring: K items land on the slots V items left and vice versa");
  constexpr int XROWS = DT * 8 + 4;  // exchange rows per wave: O registers, m and l of its two queries per lane
  constexpr int OSTRIDE = D + 4;     // fp32 staging row stride (floats), bank-spread
  static_assert(XROWS * 64 >= 32 * OSTRIDE, "the staging rows of a query half overlay its exchange area");
  constexpr int kEpilogueBytes = 2 * XROWS * 64 * 4;
  constexpr int kSmem = kSlots * T::kBytes > kEpilogueBytes ? kSlots * T::kBytes : kEpilogueBytes;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kSmem];
  constexpr int kOrdSlots = 4;                       // order entries of tile e live in slot e % 4
  constexpr int QD = LEAD + (RASTER ? 2 : 0);        // block ids are queued this many tiles ahead
  constexpr int kBias = 1024 * (kDma - 1);           // keeps the per-lane global offsets of the DMA non-negative
  __shared__ __attribute__((aligned(256))) int ord_ring[RASTER ? kOrdSlots * kBlock : 1];

  const int work = xcd_contiguous_id(blockIdx.x, per_xcd);
  if (work >= total) return;  // whole workgroup leaves before any barrier
  const long long head = work / nb;
  // which query block of the head this workgroup takes: its slot number, or what the caller's work order puts
  // there (longest lists first: workgroups that run together then have lists of similar length, their sweeps
  // over the head's K/V stay together in L2, and the last round of the launch is made of the shortest lists)
  int i = work % nb;
  if (work_order) i = min(max(work_order[work], 0), nb - 1);
  const long long row_id = head * nb + i;
  const long long head_off = head * (long long)nb * kBlock * D;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction; keep it scalar
  const int qh = wave & 1, kh = wave >> 1;
  const int c16 = lane & 15, G = lane >> 4;  // MFMA lane coordinates: column / row within a 16-row group, group
  const int n_list = min(max(cnt[row_id], 0), kmax);  // device contents are not trusted with addresses:
  const int32_t* list = idx + row_id * kmax;
  // valid query rows of this block: the first nq of its 64 positions hold tokens
  int nq = min(kBlock, max(0, Nv - i * kBlock));
  if constexpr (RASTER)
    if (ras.block_valid) nq = min(kBlock, max(0, ras.block_valid[i]));
  const uint16_t* kbase = k + head_off;
  const uint16_t* vbase = v + head_off;
  // raster mode: byte bases of this (batch, head); the K/V ones are lowered by kBias (see kc/vc below)
  long long ras_off = 0, ras_out = 0;
  if constexpr (RASTER) {
    const long long b = head / ras.Hh, h = head - b * ras.Hh;
    ras_off = b * ras.batch + h * ras.head;
    ras_out = b * ras.o_batch + h * ras.o_head;
  }
  const unsigned char* kbase_r = reinterpret_cast<const unsigned char*>(k) + ras_off - kBias;
  const unsigned char* vbase_r = reinterpret_cast<const unsigned char*>(v) + ras_off - kBias;

  // DMA plan of this wave: instruction `it` fills LDS bytes [a*1024, a*1024+1024) of a tile slot,
  // a = wave*kDma + it; lane -> (row, stored chunk position p); it fetches global chunk
  // p ^ swz(row) of that row.  The byte offsets are loop invariant; the 1024*it that the
  // instruction offset adds on both sides is taken out of the global one here.
  int kofs[kDma], vofs[kDma];
#pragma unroll
  for (int it = 0; it < kDma; ++it) {
    const int row = (wave * kDma + it) * T::kRowsPerDma + lane / T::kChunks, p = lane % T::kChunks;
    kofs[it] = (row * D + ((p ^ T::k_swz(row)) << 3)) * 2 - 1024 * it;
    vofs[it] = (row * D + ((p ^ T::v_swz(row)) << 3)) * 2 - 1024 * it;
  }
  const unsigned wave_lds = lds_address(smem) + wave * kDma * 1024;
  // raster mode: per-lane constants of the DMA offsets (chunk within the row, the bias, the 1024*it that the
  // instruction offset adds); the row part comes from the order entries of the tile
  int kc[kDma], vc[kDma], rowoff[kDma];
  if constexpr (RASTER) {
#pragma unroll
    for (int it = 0; it < kDma; ++it) {
      const int row = (wave * kDma + it) * T::kRowsPerDma + lane / T::kChunks, p = lane % T::kChunks;
      kc[it] = ((p ^ T::k_swz(row)) << 4) + kBias - 1024 * it;
      vc[it] = ((p ^ T::v_swz(row)) << 4) + kBias - 1024 * it;
      rowoff[it] = 0;
    }
  }
  // this wave's 16 order entries of tile `e` (block j) -> its part of ord_ring slot e % 4
  auto issue_ord = [&](int j, int e) {
    if constexpr (RASTER) {
      if (lane < 16) {
        const unsigned dst = lds_address(ord_ring) + ((e % kOrdSlots) * kBlock + wave * 16) * 4;
        const int32_t* src = ras.order + (long long)j * kBlock + wave * 16;
        const int voff = lane * 4;
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2" : : "s"(dst), "v"(voff), "s"(src) : "memory");
      }
    }
  };
  // rowoff[it] = byte offset of the token row that DMA instruction `it` of this lane fetches for tile e
  auto read_ord = [&](int e) {
    if constexpr (RASTER) {
      const int* slot = ord_ring + (e % kOrdSlots) * kBlock + wave * 16 + lane / T::kChunks;
#pragma unroll
      for (int it = 0; it < kDma; ++it) rowoff[it] = slot[it * T::kRowsPerDma] * (int)ras.tok;
    }
  };
  auto issue_k = [&](int j, int slot) {
    if constexpr (RASTER) {
      int off[kDma];
#pragma unroll
      for (int it = 0; it < kDma; ++it) off[it] = rowoff[it] + kc[it];
      dma_tile<kDma>(kbase_r, off, wave_lds + slot * T::kBytes);
    } else {
      dma_tile<kDma>(kbase + (long long)j * kBlock * D, kofs, wave_lds + slot * T::kBytes);
    }
  };
  auto issue_v = [&](int j, int slot) {
    if constexpr (RASTER) {
      int off[kDma];
#pragma unroll
      for (int it = 0; it < kDma; ++it) off[it] = rowoff[it] + vc[it];
      dma_tile<kDma>(vbase_r, off, wave_lds + slot * T::kBytes);
    } else {
      dma_tile<kDma>(vbase + (long long)j * kBlock * D, vofs, wave_lds + slot * T::kBytes);
    }
  };

  // The index list lives in a VGPR, 64 entries at a time (lane t holds entry 64*chunk + t), and is
  // read with v_readlane: one instruction per tile and no scalar-memory wait, which would also be
  // a wait for every LDS read in flight.
  // (read for every lane below kmax, whatever the count says, so that this load does not wait for the count's)
  const int list_raw = lane < kmax ? list[lane] : 0;
  int list_v = lane < n_list ? min(max(list_raw, 0), nb - 1) : 0;  // ... ids are clamped into [0, nb)
  auto list_at = [&](int n) { return __builtin_amdgcn_readlane(list_v, n & 63); };
  // raster mode: the valid keys of every listed block travel beside its id (lane t: block of entry t), either
  // looked up in the per-block counts (one cube per block, cut cubes padded) or, without them, what the first
  // Nv positions leave of the block
  int valid_v = kBlock;
  auto load_valid = [&]() {
    if constexpr (RASTER)
      valid_v = ras.block_valid ? min(kBlock, max(0, ras.block_valid[list_v])) : min(kBlock, max(0, Nv - list_v * kBlock));
  };
  load_valid();
  auto valid_at = [&](int n) { return __builtin_amdgcn_readlane(valid_v, n & 63); };

  // ring item 2n = K(list[n]) -> slot (2n) % SLOTS, item 2n+1 = V(list[n]) -> slot (2n+1) % SLOTS;
  // the first LEAD tiles are requested here
  if constexpr (RASTER) {
    // the order entries of the first LEAD + 2 tiles; the loop requests those of tile n + LEAD + 2
#pragma unroll
    for (int t = 0; t < LEAD + 2; ++t)
      if (t < n_list) issue_ord(list_at(t), t);
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0); each wave reads only what it requested itself
  }
#pragma unroll
  for (int t = 0; t < LEAD; ++t)
    if (t < n_list) {
      const int j = list_at(t);
      read_ord(t);
      issue_k(j, (2 * t) % kSlots);
      issue_v(j, (2 * t + 1) % kSlots);
    }
  int jq[QD + 1];  // block ids of tiles n .. n+QD (entries beyond the list read as block 0, unused)
  int nkq[QD + 1]; // raster mode: their valid key counts
#pragma unroll
  for (int t = 0; t <= QD; ++t) {
    jq[t] = list_at(t);
    nkq[t] = kBlock;
  }

  // Q fragments: for query tile nt the lane holds query row 32*qh + 16*nt + c16, channels 32 t + 8 G .. + 8
  // for every k-step t
  bf16x8 qf[2][KS];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int qrow = i * kBlock + qh * 32 + 16 * nt + c16;
    const uint16_t* qp = q + head_off + (long long)qrow * D + G * 8;
    if constexpr (RASTER)
      qp = reinterpret_cast<const uint16_t*>(reinterpret_cast<const unsigned char*>(q) + ras_off +
                                             (long long)ras.order[qrow] * ras.tok) + G * 8;
#pragma unroll
    for (int t = 0; t < KS; ++t) qf[nt][t] = *reinterpret_cast<const bf16x8*>(qp + t * 32);
    if constexpr (RASTER) {
      // padding positions have no token: their query rows are zero, as in a gathered copy (their lanes
      // take part in the wave-wide rescale decisions, so what they hold is not quite without effect)
      if (qh * 32 + 16 * nt + c16 >= nq) {
#pragma unroll
        for (int t = 0; t < KS; ++t)
#pragma unroll
          for (int e = 0; e < 8; ++e) qf[nt][t][e] = (__bf16)0.0f;
      }
    }
  }

  // O^T accumulators: quarter dt % 4 of o[nt][dt / 4], element r = channel 16 dt + 4 G + r of query 32 qh + 16 nt + c16
  constexpr int OT = (DT + 3) / 4;
  f32x16 o[2][OT];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int k = 0; k < OT; ++k)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[nt][k][r] = 0.f;
  // per query tile nt (this lane's two queries); each is identical in the four lanes of its query
  float m[2] = {-INFINITY, -INFINITY};  // running reference max (log2 domain)
  float l[2] = {0.f, 0.f};              // this lane's partial row sum (its 8 keys per tile)
  // derived from m, refreshed only when m moves (rare): the exponent offset and the raise threshold
  float neg_m[2] = {0.f, 0.f};                  // -m - p_shift, or 0 while every key seen so far was masked (m = -inf)
  float m_raise[2] = {-INFINITY, -INFINITY};    // m + kRescaleSlack

  // per-lane LDS byte offsets of the fragment reads (loop invariant)
  // K fragment of key tile mt, k-step t: key row 32 kh + 16 mt + c16, chunk 4 t + G; +16 rows is a constant
  // (both tables are XOR patterns: kfrag[t] = kfrag[0] ^ (t << 6) and vfrag[dt] = vfrag[0] ^ (dt << 5), because the
  // swizzles only touch address bits that t and dt alone set.  The three-workgroup shape has no registers to
  // spare and derives the entries with one v_xor per use; the other shapes keep them in registers.)
  constexpr bool kLean = WGS >= 3;
  int kfrag[KS];
#pragma unroll
  for (int t = 0; t < KS; ++t) kfrag[t] = T::k_off(kh * 32 + c16, 4 * t + G);
  // V^T fragment of d sub-tile dt: contraction slots 0..3 are keys 4 G + (0..3), slots 4..7 keys
  // 16 + 4 G + (0..3) of this wave's half (the order the S^T accumulators hold them); the 16 lanes of a
  // group address the 4 key rows x 16 channels that the transposing read hands out column by column
  int vfrag[DT];
  {
    const int key0 = kh * 32 + 4 * G + (c16 >> 2);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const int dcol = 16 * dt + 4 * (c16 & 3);  // 4 channels = half a chunk
      vfrag[dt] = T::v_off(key0, dcol >> 3) + ((dcol >> 2) & 1) * 8;
    }
  }

  __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): the first tiles and Q have landed
  if constexpr (RASTER) {  // (read here, behind the wait that everything shares: an earlier read would hold the Q loads back)
#pragma unroll
    for (int t = 0; t <= QD; ++t) nkq[t] = valid_at(t);
  }
  // pin the Q fragments here: otherwise the compiler sinks their loads into the loop and then waits
  // for "all outstanding loads" there, which would also wait for the tile prefetch it cannot see
#pragma unroll
  for (int t = 0; t < KS; ++t) asm volatile("" ::"v"(qf[0][t]), "v"(qf[1][t]));
  __syncthreads();

  // One tile.  PHASE = n % SLOTS is a compile-time constant so that every LDS offset of the ring
  // folds into the instruction.  On entry K(n) is in LDS and visible to every wave and the slot of
  // V(n-1) is free.  A freed slot of item e is refilled with item e + SLOTS.  STEADY (compile time)
  // says that tile n+LEAD exists, which spares the main loop every end-of-list check.
  // blocks from this one on hold padded keys: the partial block (if Nv is not a multiple of 64) and, when the
  // tensors are padded by whole blocks, every block behind it.  A caller's list may name those too: all of
  // their keys are masked, as the masked-attention equation has it (they then add nothing to the row).
  // (raster mode carries the valid key count of every listed block in nkq instead)
  const int first_padded_j = Nv / kBlock;
  auto tile_step = [&](auto phase_c, auto steady_c, int n) {
    constexpr int phase = decltype(phase_c)::value;
    constexpr int kslot = (2 * phase) % kSlots, vslot = (2 * phase + 1) % kSlots;
    constexpr int freed_v = (2 * phase + kSlots - 1) % kSlots;  // slot of item 2n-1 = V(n-1)
    const int j = jq[0];
    const int j_pre = jq[LEAD];
    const bool steady = decltype(steady_c)::value || n + LEAD < n_list;
    if constexpr (RASTER) {
      // per tile and wave: one order request (tile n+LEAD+2), then K (kDma), then V (kDma)
      if (decltype(steady_c)::value || n + LEAD + 2 < n_list) issue_ord(jq[QD], n + LEAD + 2);
      if (steady) read_ord(n + LEAD);
    }
    if (steady) issue_k(j_pre, freed_v);  // item 2n-1+SLOTS = K(n+LEAD)

    // ---- S^T = K Q^T over this wave's 32 keys x 32 queries: s[mt][nt] --------------------------
    f32x16 s;  // quarter 2 mt + nt = tile (mt, nt)
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
    {
      // fragments are read in batches and awaited once per batch: every s_waitcnt costs the
      // wave an issue slot, and the other waves of the SIMD cover the LDS latency
      const unsigned char* kb = smem + kslot * T::kBytes;
      if constexpr (kLean) asm volatile("" : "+v"(kfrag[0]));  // keeps the XORs in the loop (hoisted, they are the table again)
      constexpr int KB = WGS <= 2 ? KS : 1;  // k-steps per batch (register budget)
#pragma unroll
      for (int t0 = 0; t0 < KS; t0 += KB) {
        bf16x8 kf[KB][2];
#pragma unroll
        for (int t = 0; t < KB; ++t)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
            kf[t][mt] = *reinterpret_cast<const bf16x8*>(kb + (kLean ? kfrag[0] ^ ((t0 + t) << 6) : kfrag[t0 + t]) +
                                                         mt * 16 * T::kRowBytes);
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
        // the fences keep each batch together: reads, one wait, back-to-back MFMAs
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < KB; ++t)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
              set_quarter(s, 2 * mt + nt,
                          __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][mt], qf[nt][t0 + t], quarter(s, 2 * mt + nt), 0, 0, 0));
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // V(n) has landed; only the SLOTS-2 items requested after it may still be in flight (near the
    // end of the list fewer are, so the last LEAD tiles simply wait for everything)
    // (raster mode: what this wave requested after V(n) is LEAD-1 whole tiles' worth of 2 kDma + 1
    // requests plus this tile's order and K requests)
    constexpr int kMidWait = RASTER ? (LEAD - 1) * (2 * kDma + 1) + kDma + 1 : (kSlots - 2) * kDma;
    if (RASTER ? decltype(steady_c)::value : steady)  // raster: the request counts only hold in whole rounds
      __builtin_amdgcn_s_waitcnt(0x0f70 | kMidWait);
    else
      __builtin_amdgcn_s_waitcnt(0x0f70);
    __syncthreads();  // ... for every wave; and nobody reads K(n) any more
    if (steady) issue_v(j_pre, kslot);  // item 2n+SLOTS = V(n+LEAD) takes K(n)'s slot
    // block ids for the next iteration: shift the queue and append tile n+1+LEAD
    const int nk = nkq[0];
#pragma unroll
    for (int t = 0; t < QD; ++t) {
      jq[t] = jq[t + 1];
      nkq[t] = nkq[t + 1];
    }
    if (((n + 1 + QD) & 63) == 0) {  // next 64 entries; awaited right here (once per 64 tiles) so that
      list_v = n + 1 + QD + lane < n_list ? min(max(list[n + 1 + QD + lane], 0), nb - 1) : 0;  // the hot path carries no
      __builtin_amdgcn_s_waitcnt(0x0f70);                                  // vector-memory wait
      asm volatile("" ::"v"(list_v));
      if constexpr (RASTER) {
        load_valid();
        __builtin_amdgcn_s_waitcnt(0x0f70);
        asm volatile("" ::"v"(valid_v));
      }
    }
    jq[QD] = list_at(n + 1 + QD);
    if constexpr (RASTER) nkq[QD] = valid_at(n + 1 + QD);

    // s[8 mt + 4 nt + r] of lane (c16, G) is key 32 kh + 16 mt + 4 G + r of the tile, query 32 qh + 16 nt + c16
    if (RASTER ? nk < kBlock : j >= first_padded_j) {
      // valid keys of the tile ahead of this lane's first
      const int lim = (RASTER ? nk : Nv - j * kBlock) - (kh * 32 + 4 * G);
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int r = 0; r < 4; ++r) s[8 * mt + 4 * nt + r] = (16 * mt + r) < lim ? s[8 * mt + 4 * nt + r] : -INFINITY;
    }

    // ---- online softmax (log2 domain, lazily raised reference max) -------------------------
    // The raise test needs no cross-lane step: if no lane holds a value above its query's threshold,
    // no query has one.  Only a raise itself (rare) takes the maximum over the four lanes of a query.
    float mx[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
      mx[nt] = max8(s[4 * nt], s[4 * nt + 1], s[4 * nt + 2], s[4 * nt + 3], s[8 + 4 * nt], s[8 + 4 * nt + 1],
                    s[8 + 4 * nt + 2], s[8 + 4 * nt + 3]) * scale_log2e;
    if (__any(mx[0] > m_raise[0] || mx[1] > m_raise[1])) {  // wave-uniform; always taken on the first live tile
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const float m_new = fmaxf(m[nt], max_over_groups(mx[nt]));
        const float alpha = fast_exp2(m[nt] - (m_new == -INFINITY ? 0.f : m_new));  // m = -inf -> 0
        m[nt] = m_new;
        neg_m[nt] = m_new == -INFINITY ? 0.f : -m_new - p_shift;
        m_raise[nt] = m_new + kRescaleSlack;
        l[nt] *= alpha;
#pragma unroll
        for (int k = 0; k < OT; ++k)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[nt][k][r] *= alpha;
      }
    }
    // P^T of this wave's 32 keys, rounded to bf16 and packed two per register: per query the same four
    // registers feed the row sum (v_dot2 with ones) and, as they stand, the B operand of the second product
    typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned uint4v;
    bf16x8 pf[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      bf16x2 pk[4];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 4; r += 2) {
          pk[2 * mt + (r >> 1)][0] = (__bf16)fast_exp2(fmaf(s[8 * mt + 4 * nt + r], scale_log2e, neg_m[nt]));
          pk[2 * mt + (r >> 1)][1] = (__bf16)fast_exp2(fmaf(s[8 * mt + 4 * nt + r + 1], scale_log2e, neg_m[nt]));
        }
      // the row sum is taken over the ROUNDED probabilities, the ones P V actually uses, so that
      // the final division cancels the rounding of a dominant key instead of keeping it
      bf16x2 ones;
      ones[0] = (__bf16)1.0f;
      ones[1] = (__bf16)1.0f;
#pragma unroll
      for (int r = 0; r < 4; ++r) l[nt] = __builtin_amdgcn_fdot2_f32_bf16(pk[r], ones, l[nt], false);
      const uint4v w = {__builtin_bit_cast(unsigned, pk[0]), __builtin_bit_cast(unsigned, pk[1]),
                        __builtin_bit_cast(unsigned, pk[2]), __builtin_bit_cast(unsigned, pk[3])};
      pf[nt] = __builtin_bit_cast(bf16x8, w);
    }

    // ---- O^T += V^T P^T: one MFMA per (d sub-tile, query tile), its 32 contraction slots = this wave's keys ----
    {
      const unsigned char* vb = smem + vslot * T::kBytes;
      if constexpr (kLean) asm volatile("" : "+v"(vfrag[0]));
      constexpr int VB = WGS <= 2 ? DT : 2;  // d sub-tiles per batch
#pragma unroll
      for (int dt0 = 0; dt0 < DT; dt0 += VB) {
        bf16x8 vf[VB];
#pragma unroll
        for (int dd = 0; dd < VB; ++dd) {
          const unsigned char* p = vb + (kLean ? vfrag[0] ^ ((dt0 + dd) << 5) : vfrag[dt0 + dd]);
          const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)p);
          const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (short4v __attribute__((address_space(3)))*)(p + 16 * T::kRowBytes));
          const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          __builtin_memcpy(&vf[dd], &both, sizeof(bf16x8));
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int dd = 0; dd < VB; ++dd)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt)
            set_quarter(o[nt][(dt0 + dd) >> 2], (dt0 + dd) & 3,
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dd], pf[nt], quarter(o[nt][(dt0 + dd) >> 2], (dt0 + dd) & 3), 0, 0, 0));
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // pin each accumulator tuple to one 16-register unit once per tile (see quarter())
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int k = 0; k < OT; ++k) asm volatile("" : "+v"(o[nt][k]));

    // K(n+1) has landed; again at most SLOTS-2 younger items are in flight
    constexpr int kEndWait = RASTER ? (LEAD - 1) * (2 * kDma + 1) + kDma : (kSlots - 2) * kDma;
    if (RASTER ? decltype(steady_c)::value : steady)
      __builtin_amdgcn_s_waitcnt(0x0f70 | kEndWait);
    else
      __builtin_amdgcn_s_waitcnt(0x0f70);
    __syncthreads();  // ... for every wave; and nobody reads V(n) any more
  };
  {
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using P2 = std::integral_constant<int, 2>;
    using P3 = std::integral_constant<int, 3>;
    using P4 = std::integral_constant<int, 4>;
    int n = 0;
    for (; n + kSlots + LEAD <= n_list; n += kSlots) {  // whole rounds of the ring, no end-of-list checks
      tile_step(P0{}, std::true_type{}, n);
      tile_step(P1{}, std::true_type{}, n + 1);
      tile_step(P2{}, std::true_type{}, n + 2);
      if constexpr (kSlots >= 5) {
        tile_step(P3{}, std::true_type{}, n + 3);
        tile_step(P4{}, std::true_type{}, n + 4);
      }
    }
    // the last, partial round (n is a multiple of SLOTS here, so the phases line up)
    if (n < n_list) tile_step(P0{}, std::false_type{}, n);
    if (n + 1 < n_list) tile_step(P1{}, std::false_type{}, n + 1);
    if (n + 2 < n_list) tile_step(P2{}, std::false_type{}, n + 2);
    if constexpr (kSlots >= 5) {
      if (n + 3 < n_list) tile_step(P3{}, std::false_type{}, n + 3);
      if (n + 4 < n_list) tile_step(P4{}, std::false_type{}, n + 4);
    }
    // up to SLOTS + LEAD - 1 tiles can remain: LEAD - 1 more
    static_assert(LEAD <= 2, "one extra tile after the partial round");
    if constexpr (LEAD == 2) {
      if (n + kSlots < n_list) tile_step(P0{}, std::false_type{}, n + kSlots);
    }
  }

  // ---- merge the two key halves, stage the block row-major in LDS, store coalesced ----------
  // (the loop ended with a barrier, so the tile slots are free).  The staging rows of a query half
  // overlay the exchange area that the SAME wave has just read into registers.
  float l_row[2];  // this wave's row sums: over the four lanes of each query
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) l_row[nt] = sum_over_groups(l[nt]);
  float* xch = reinterpret_cast<float*>(smem) + qh * XROWS * 64;  // [XROWS][64 lanes] of this query half
  if (kh == 1) {
    float* dst = xch + lane;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 4; ++r) dst[((dt * 2 + nt) * 4 + r) * 64] = o[nt][dt >> 2][4 * (dt & 3) + r];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      dst[(DT * 8 + nt) * 64] = m[nt];
      dst[(DT * 8 + 2 + nt) * 64] = l_row[nt];
    }
  }
  __syncthreads();
  if (kh == 0) {
    const float* src = xch + lane;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const float m1 = src[(DT * 8 + nt) * 64], l1 = src[(DT * 8 + 2 + nt) * 64];
      const float mm = fmaxf(m[nt], m1);
      const float m_ref = mm == -INFINITY ? 0.f : mm;
      const float a0 = fast_exp2(m[nt] - m_ref), a1 = fast_exp2(m1 - m_ref);
      const float lt = l_row[nt] * a0 + l1 * a1;
      const int row = qh * 32 + 16 * nt + c16, token = i * kBlock + row;
      const bool live = row < nq && lt > 0.f;  // lt == 0: empty list, or every listed key is padding
      const float inv = live ? 1.f / lt : 0.f;
      const float w0 = live ? a0 * inv : 0.f, w1 = live ? a1 * inv : 0.f;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float val = o[nt][dt >> 2][4 * (dt & 3) + r] * w0 + src[((dt * 2 + nt) * 4 + r) * 64] * w1;
          o[nt][dt >> 2][4 * (dt & 3) + r] = live ? val : 0.f;
        }
      if (lse && G == 0) {
        const float val = live ? (mm + p_shift + __log2f(lt)) * kLn2 : -INFINITY;
        if constexpr (RASTER) {  // [B, Hh, Nv] in raster order; padded rows have no place there
          if (row < nq) lse[head * (long long)Nv + ras.order[token]] = val;
        } else {
          lse[head * (long long)nb * kBlock + token] = val;
        }
      }
    }
    // every exchange value of this wave must be in registers before its area is overwritten
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      float* stage = xch + (16 * nt + c16) * OSTRIDE;  // row 32 qh + 16 nt + c16 of the block
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {  // quarter dt % 4 of o[nt][dt / 4] is channels 16 dt + 4 G .. + 3
        const f32x16& t = o[nt][dt >> 2];
        const int e = 4 * (dt & 3);
        *reinterpret_cast<float4*>(stage + 16 * dt + 4 * G) = make_float4(t[e], t[e + 1], t[e + 2], t[e + 3]);
      }
    }
  }
  __syncthreads();
  {
    // 64 rows x D channels, 4 channels per thread per pass, consecutive threads -> consecutive addresses
    const float* stage = reinterpret_cast<const float*>(smem);  // row r at (r / 32) * XROWS * 64 + (r % 32) * OSTRIDE
    constexpr int PIECES = kBlock * D / 4;
    const long long blk_off = head_off + (long long)i * kBlock * D;
#pragma unroll
    for (int it = 0; it < PIECES / kThreads; ++it) {
      const int id = it * kThreads + tid;
      const int row = id / (D / 4), c4 = (id % (D / 4)) * 4;
      float4 val = *reinterpret_cast<const float4*>(stage + (row >> 5) * (XROWS * 64) + (row & 31) * OSTRIDE + c4);
      if (fuse.coarse && row < nq) {
        // second branch folded into the store: out = gate_fine * attention + gate_coarse * cube-level row of this cube
        const float4 cz = *reinterpret_cast<const float4*>(fuse.coarse + (head * nb + i) * (long long)D + c4);
        float4 gf = make_float4(1.f, 1.f, 1.f, 1.f), gc = gf;
        long long gate_off = blk_off + row * D + c4;  // in elements
        if constexpr (RASTER)  // the gates are raster tensors laid out like q
          gate_off = (ras_off + (long long)ras.order[i * kBlock + row] * ras.tok) / 2 + c4;
        if (fuse.gate_fine) gf = load_bf16x4(fuse.gate_fine + gate_off);
        if (fuse.gate_coarse) gc = load_bf16x4(fuse.gate_coarse + gate_off);
        val.x = fmaf(gf.x, val.x, gc.x * cz.x);
        val.y = fmaf(gf.y, val.y, gc.y * cz.y);
        val.z = fmaf(gf.z, val.z, gc.z * cz.z);
        val.w = fmaf(gf.w, val.w, gc.w * cz.w);
      }
      void* dst;
      if constexpr (RASTER) {
        if (row >= nq) continue;  // the raster tensor has no padded rows
        dst = static_cast<unsigned char*>(out) + ras_out + (long long)ras.order[i * kBlock + row] * ras.o_tok +
              c4 * (OUT_F32 ? 4 : 2);
      } else {
        dst = OUT_F32 ? static_cast<void*>(static_cast<float*>(out) + blk_off + row * D + c4)
                      : static_cast<void*>(static_cast<uint16_t*>(out) + blk_off + row * D + c4);
      }
      // stream_out (the launcher's choice, the same for every workgroup): streaming stores.  The output is not read
      // again by this launch, and written the ordinary way its lines push K/V tiles out of the L2.
      if (OUT_F32) {
        f32x4 vv = {val.x, val.y, val.z, val.w};
        if (stream_out)
          __builtin_nontemporal_store(vv, reinterpret_cast<f32x4*>(dst));
        else
          *reinterpret_cast<f32x4*>(dst) = vv;
      } else {
        bf16x4 pk;
        pk[0] = (__bf16)val.x; pk[1] = (__bf16)val.y; pk[2] = (__bf16)val.z; pk[3] = (__bf16)val.w;
        if (stream_out)
          __builtin_nontemporal_store(pk, reinterpret_cast<bf16x4*>(dst));
        else
          *reinterpret_cast<bf16x4*>(dst) = pk;
      }
    }
  }
}

template <int D, bool OUT_F32, int SLOTS, int WGS, bool RASTER = false>
hipError_t run(const void* q, const void* k, const void* v, const Dims& s, const int32_t* idx, const int32_t* cnt,
               int kmax, float scale, void* out, float* lse, const FuseArgs& fuse, hipStream_t st,
               const RasterArgs& ras = RasterArgs{}, const int32_t* work_order = nullptr) {
  const long long total = s.bh() * s.nb;
  const int per_xcd = (int)((total + kNumXcd - 1) / kNumXcd);
  const unsigned grid = (unsigned)per_xcd * kNumXcd;
  const float sl2 = scale * kLog2e;
  // tau = 2^-(kDropLog2 + ceil(log2(keys of the longest list))), p_shift = 126 + log2(tau), kept within [64, 110]
  int bits = 0;
  while ((1LL << bits) < (long long)kmax * kBlock) ++bits;
  const float p_shift = (float)(126 - kDropLog2 - bits < 64 ? 64 : 126 - kDropLog2 - bits > 110 ? 110 : 126 - kDropLog2 - bits);
  auto Q = static_cast<const uint16_t*>(q);
  auto K = static_cast<const uint16_t*>(k);
  auto V = static_cast<const uint16_t*>(v);
  // Streaming output stores where the L2 has something to lose: measured -1 % at the 480p shape (a head's K and V:
  // 16.8 MB), -2.7 % with ragged budgets at 16384 tokens, nothing on dense lists, but +4.4 % at the 720p shape
  // (38.7 MB per head: the L2 serves a quarter of the tile requests there whatever the output does, and the launch
  // runs at the limit of the fabric, which ordinary stores load more evenly).
  const int stream_out = 2LL * s.nb * kBlock * D * 2 <= (32LL << 20);
  attn_bf16<D, OUT_F32, SLOTS, WGS, RASTER><<<grid, kThreads, 0, st>>>(Q, K, V, idx, cnt, out, lse, s.nb, s.Nv, kmax, sl2,
                                                                     p_shift, (int)total, per_xcd, fuse, ras, work_order,
                                                                     stream_out);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_bf16(const void* q, const void* k, const void* v, const Dims& s, const int32_t* idx,
                            const int32_t* cnt, int kmax, float scale, void* out, bool out_f32, float* lse,
                            const FuseArgs& fuse, hipStream_t st, const int32_t* work_order) {
  // Two launch shapes, both with a 3-slot ring (48 KiB at d = 128), chosen by measurement at the 480p shape:
  //   sparse lists: 2 workgroups per CU with the whole register file between them, so that every fragment
  //     of a tile is read in one batch (a 5-slot ring that requests tiles two iterations ahead was 1 % slower
  //     at 51, 25 and ragged 8..64 blocks and at the 720p shape; 3 workgroups per CU with the small batches
  //     their 168 registers allow was 19 % slower);
  //   dense-like lists (at least half of the blocks kept, so neighbouring query blocks share most
  //     tiles and L2 serves them): 3 workgroups per CU, for the extra wave per SIMD (2 % faster there).
  const bool dense_like = 2 * (long long)kmax >= s.nb;
#define USV_ATTN_CASE(DD, F32)                                                                         \
  return dense_like ? run<DD, F32, 3, 3>(q, k, v, s, idx, cnt, kmax, scale, out, lse, fuse, st, RasterArgs{}, work_order) \
                    : run<DD, F32, 3, 2>(q, k, v, s, idx, cnt, kmax, scale, out, lse, fuse, st, RasterArgs{}, work_order)
  if (s.d == 128) {
    if (out_f32) USV_ATTN_CASE(128, true);
    USV_ATTN_CASE(128, false);
  }
  if (out_f32) USV_ATTN_CASE(64, true);
  USV_ATTN_CASE(64, false);
#undef USV_ATTN_CASE
}

// Raster-order tensors: the sparse shape (3-slot ring, 2 workgroups per CU) plus the order ring.
hipError_t launch_attn_bf16_raster(const void* q, const void* k, const void* v, const Dims& s, const RasterArgs& ras,
                                   const int32_t* idx, const int32_t* cnt, int kmax, float scale, void* out,
                                   bool out_f32, float* lse, const FuseArgs& fuse, hipStream_t st,
                                   const int32_t* work_order) {
#define USV_RASTER_CASE(DD, F32) \
  return run<DD, F32, 3, 2, true>(q, k, v, s, idx, cnt, kmax, scale, out, lse, fuse, st, ras, work_order)
  if (s.d == 128) {
    if (out_f32) USV_RASTER_CASE(128, true);
    USV_RASTER_CASE(128, false);
  }
  if (out_f32) USV_RASTER_CASE(64, true);
  USV_RASTER_CASE(64, false);
#undef USV_RASTER_CASE
}

}  // namespace usv
