// Raster <-> cube-major token order (paper Figure 2, right: tokens are partitioned into 3-D cubes
// on the way into the sparse attention and broadcast back to the token grid on the way out).
//
// Pure data movement, HBM bound: every token row (d channels) is read once and written once.
// One workgroup moves 64 consecutive RASTER tokens of one (batch, head): the first 64 lanes turn
// their raster index into its cube-major position (closed form, a handful of integer divisions),
// then all lanes copy the rows 16 bytes at a time.  Consecutive raster tokens run along w, so
// the raster side is contiguous and the cube side comes in runs of cw rows (>= 256 bytes each).
// Measured on MI355X (working set cycled beyond the Infinity Cache): at most four 16-byte pieces
// per lane (8 per lane: 3.7 instead of 5.5 TB/s), source read with non-temporal loads (it is dead
// afterwards; +3 %); the destination is stored normally because the next kernel reads it (streaming
// stores make this kernel 8 % faster but its consumer slower by as much).
#include "usv_internal.h"

namespace usv {

// Cube-major position of raster token (t, h, w).  Whole cubes come first, one per 64-token block, in
// raster order of their cube coordinates; the cubes the boundary cuts follow in the same order, packed.
__host__ __device__ static inline int imin(int a, int b) { return a < b ? a : b; }

__host__ __device__ long long cube_position(const CubeGrid& g, int t, int h, int w) {
  const int it = t / g.ct, ih = h / g.ch, iw = w / g.cw;
  const int lt = t - it * g.ct, lh = h - ih * g.ch, lw = w - iw * g.cw;
  if (it < g.Tf && ih < g.Hf && iw < g.Wf)
    return (long long)kBlock * (((long long)it * g.Hf + ih) * g.Wf + iw) + (lt * g.ch + lh) * g.cw + lw;
  // extents of this (cut) cube
  const int et = imin(g.ct, g.T - it * g.ct), eh = imin(g.ch, g.H - ih * g.ch), ew = imin(g.cw, g.W - iw * g.cw);
  // tokens of every cube that precedes this one in raster order of cube coordinates: whole slabs of
  // ct frames, then whole bands of ch rows inside this slab, then the cubes to the left in this band
  const long long before = (long long)it * g.ct * g.H * g.W + (long long)et * ((long long)ih * g.ch * g.W + (long long)eh * iw * g.cw);
  // ... of which this many are whole cubes (64 tokens each), already placed in the first part
  long long whole_before;
  if (it < g.Tf)
    whole_before = (long long)it * g.Hf * g.Wf + (ih < g.Hf ? (long long)ih * g.Wf + imin(iw, g.Wf) : (long long)g.Hf * g.Wf);
  else
    whole_before = (long long)g.Tf * g.Hf * g.Wf;
  const long long n_whole = (long long)g.Tf * g.Hf * g.Wf;
  return kBlock * n_whole + (before - kBlock * whole_before) + (lt * eh + lh) * ew + lw;
}

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned chunk_t;  // 16 bytes

// GATHER: raster -> cube (and zero the padding rows); otherwise cube -> raster.
// CHUNKS = 16-byte pieces per token row.
template <bool GATHER, int CHUNKS>
__global__ __launch_bounds__(CHUNKS >= 32 ? 512 : 256) void cube_move(const unsigned char* __restrict__ src,
                                                      unsigned char* __restrict__ dst, CubeGrid g, int N, int Nv,
                                                      int Hh, long long sb, long long sh, long long st) {
  constexpr int kThreads = CHUNKS >= 32 ? 512 : 256;  // <= 4 pieces per lane
  __shared__ int pos[kBlock];
  const int tid = threadIdx.x;
  const int r0 = blockIdx.x * kBlock;
  const int bh = blockIdx.y, b = bh / Hh, head = bh - b * Hh;
  if (tid < kBlock) {
    const int r = r0 + tid;
    int p = r;  // padding rows keep their place
    if (r < Nv) {
      const int hw = g.H * g.W;
      const int t = r / hw, rem = r - t * hw, h = rem / g.W, w = rem - h * g.W;
      p = (int)cube_position(g, t, h, w);
    }
    pos[tid] = p;
  }
  __syncthreads();
  constexpr int kRowBytes = CHUNKS * 16;
  constexpr int PER_THREAD = kBlock * CHUNKS / kThreads;
  static_assert(kBlock * CHUNKS % kThreads == 0, "whole passes");
  const unsigned char* raster_c = GATHER ? src : nullptr;
  unsigned char* raster_m = GATHER ? nullptr : dst;
  const long long raster_base = (long long)b * sb + (long long)head * sh;  // bytes
  const long long cube_base = (long long)bh * N * kRowBytes;
  chunk_t val[PER_THREAD];
  // loads first (all in flight together), then stores
#pragma unroll
  for (int it = 0; it < PER_THREAD; ++it) {
    const int c = it * kThreads + tid, row = c / CHUNKS, ch = c - row * CHUNKS, r = r0 + row;
    val[it] = chunk_t{0u, 0u, 0u, 0u};
    if (r < Nv) {
      const unsigned char* p = GATHER ? raster_c + raster_base + (long long)r * st + ch * 16
                                      : src + cube_base + (long long)pos[row] * kRowBytes + ch * 16;
      val[it] = __builtin_nontemporal_load(reinterpret_cast<const chunk_t*>(p));
    }
  }
#pragma unroll
  for (int it = 0; it < PER_THREAD; ++it) {
    const int c = it * kThreads + tid, row = c / CHUNKS, ch = c - row * CHUNKS, r = r0 + row;
    if (GATHER) {
      if (r < N) *reinterpret_cast<chunk_t*>(dst + cube_base + (long long)pos[row] * kRowBytes + ch * 16) = val[it];
    } else {
      if (r < Nv) *reinterpret_cast<chunk_t*>(raster_m + raster_base + (long long)r * st + ch * 16) = val[it];
    }
  }
}

// order[p] = raster index of the token at cube-major position p (p < Nv), 0 for the padding positions.
__global__ __launch_bounds__(256) void cube_order(int32_t* __restrict__ order, CubeGrid g, int N, int Nv) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r < Nv) {
    const int hw = g.H * g.W;
    const int t = r / hw, rem = r - t * hw, h = rem / g.W, w = rem - h * g.W;
    order[cube_position(g, t, h, w)] = r;
  } else if (r < N) {
    order[r] = 0;
  }
}

// One cube per block, every cube (cut cubes padded): position p = 64 b + r belongs to cube b (raster order of the
// cube coordinates); its first n_b = clipped volume positions hold the cube's tokens in raster order of the local
// coordinates, the rest is padding (order = 0, a valid index; block_valid tells the kernels which rows count).
__global__ __launch_bounds__(256) void cube_order_padded(int32_t* __restrict__ order, int32_t* __restrict__ block_valid,
                                                         CubeGrid g, int n_cubes) {
  const int p = blockIdx.x * 256 + threadIdx.x;
  const int b = p / kBlock, r = p - b * kBlock;
  if (b >= n_cubes) return;
  const int nH = (g.H + g.ch - 1) / g.ch, nW = (g.W + g.cw - 1) / g.cw;
  const int it = b / (nH * nW), rem = b - it * nH * nW, ih = rem / nW, iw = rem - ih * nW;
  const int et = imin(g.ct, g.T - it * g.ct), eh = imin(g.ch, g.H - ih * g.ch), ew = imin(g.cw, g.W - iw * g.cw);
  const int n = et * eh * ew;
  if (r == 0) block_valid[b] = n;
  int v = 0;
  if (r < n) {
    const int lt = r / (eh * ew), r2 = r - lt * eh * ew, lh = r2 / ew, lw = r2 - lh * ew;
    v = ((it * g.ct + lt) * g.H + ih * g.ch + lh) * g.W + iw * g.cw + lw;
  }
  order[p] = v;
}

template <bool GATHER, int CHUNKS>
hipError_t run(const void* src, void* dst, const CubeGrid& g, const Dims& s, long long sb, long long sh, long long st,
               hipStream_t stream) {
  const dim3 grid((unsigned)(s.N / kBlock), (unsigned)s.bh());
  cube_move<GATHER, CHUNKS><<<grid, CHUNKS >= 32 ? 512 : 256, 0, stream>>>(static_cast<const unsigned char*>(src),
                                                           static_cast<unsigned char*>(dst), g, s.N, s.Nv, s.Hh, sb, sh, st);
  return hipGetLastError();
}

}  // namespace

// strides in BYTES
hipError_t launch_cube_move(bool gather, const void* src, void* dst, const CubeGrid& g, const Dims& s, long long sb,
                            long long sh, long long st, hipStream_t stream) {
  const int chunks = s.d * (s.bf16 ? 2 : 4) / 16;
#define USV_MOVE_CASE(C)                                                             \
  if (chunks == C)                                                                   \
  return gather ? run<true, C>(src, dst, g, s, sb, sh, st, stream) : run<false, C>(src, dst, g, s, sb, sh, st, stream)
  USV_MOVE_CASE(8);
  USV_MOVE_CASE(16);
  USV_MOVE_CASE(32);
#undef USV_MOVE_CASE
  return hipErrorInvalidValue;  // unreachable: the API admits d in {64, 128}, bf16 or fp32
}

hipError_t launch_cube_order(int32_t* order, const CubeGrid& g, int N, int Nv, hipStream_t stream) {
  cube_order<<<(unsigned)((N + 255) / 256), 256, 0, stream>>>(order, g, N, Nv);
  return hipGetLastError();
}

hipError_t launch_cube_order_padded(int32_t* order, int32_t* block_valid, const CubeGrid& g, hipStream_t stream) {
  const int n_cubes = ((g.T + g.ct - 1) / g.ct) * ((g.H + g.ch - 1) / g.ch) * ((g.W + g.cw - 1) / g.cw);
  cube_order_padded<<<(unsigned)((n_cubes * kBlock + 255) / 256), 256, 0, stream>>>(order, block_valid, g, n_cubes);
  return hipGetLastError();
}

}  // namespace usv
