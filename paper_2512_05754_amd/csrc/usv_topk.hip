// Stage 2: per-query-block top-k key-block selection ("top-k cube selection", paper Figure 2).
//
// One 64-lane wavefront owns one score row.  The row lives in registers (element e*64+lane in
// slot e), mapped to order-preserving unsigned keys.  The k-th largest key is found by a
// bit-by-bit search from the most significant bit (each step is a per-lane compare-and-count plus
// one wave-wide sum),
// which makes the result a pure function of the (key, index) total order: bit-exact and free of
// atomics.  Ties at the threshold are broken towards the lower block index with ballot prefix
// counts, and the survivors are written in ascending block index in one more pass.
#include "usv_internal.h"

namespace usv {
namespace {

constexpr int kRowsPerWg = 4;  // 4 wavefronts, one row each

// Order-preserving key of a canonicalised fp32: -0 == +0, NaN below everything (also -inf).
__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t b = __float_as_uint(x);
  if ((b & 0x7fffffffu) > 0x7f800000u) return 0u;  // NaN
  if (b == 0x80000000u) b = 0u;                    // -0 -> +0
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Sum of a per-lane count over the 64 lanes, as a wave-uniform value: four DPP adds leave every 16-lane row's
// total in all of its lanes (pairs, quads, then the row rotated by 4 and by 8), and the four row totals are
// read back with v_readlane.  No LDS, no ballots.
__device__ __forceinline__ int wave_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x124, 0xf, 0xf, false);  // row_ror:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false);  // row_ror:8
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
         __builtin_amdgcn_readlane(v, 48);
}

// number of set bits of `mask` below this lane
__device__ __forceinline__ int lanes_below(unsigned long long mask) {
  return __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
}

template <int EPL>  // elements per lane: row length <= 64 * EPL
__global__ __launch_bounds__(64 * kRowsPerWg) void select_topk(const float* __restrict__ scores,
                                                               const int32_t* __restrict__ budgets, int k_uniform,
                                                               int kmax, int nb, int nb_valid, long long rows,
                                                               int force_local, int32_t* __restrict__ idx,
                                                               int32_t* __restrict__ cnt) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * kRowsPerWg + (threadIdx.x >> 6);
  if (row >= rows) return;  // whole wavefront leaves together; no barriers in this kernel
  const int i = (int)(row % nb);
  int32_t* out = idx + row * kmax;

  int want = budgets ? budgets[row] : k_uniform;
  want = max(0, min(want, min(kmax, nb_valid)));
  if (i >= nb_valid) want = 0;
  want = __builtin_amdgcn_readfirstlane(want);  // the same in every lane; keep the search loop scalar

  if (want > 0) {
    const float* src = scores + row * nb;
    // every load of the row is in flight at once (slots past the row re-read its last score and are
    // overwritten below)
    float x[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) x[e] = src[min(e * 64 + lane, nb - 1)];
    uint32_t key[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const int j = e * 64 + lane;
      // slots beyond the valid blocks get the lowest key; `want <= nb_valid` and the index
      // tie-break keep them out of the result
      key[e] = j < nb_valid ? order_key(x[e]) : 0u;
      // local-cube allocation: the row's own cube gets a key above every score (order_key never
      // returns 0xffffffff), so it is kept first and the rest of the budget goes to the best others
      if (force_local && j == i) key[e] = 0xffffffffu;
    }
    // threshold = the want-th largest key among the valid slots.  Every candidate is >= 1, so the slots
    // beyond the valid blocks (key 0) never count.  The search stops as soon as a candidate splits off
    // exactly `want` keys: they are the answer whatever the lower bits are (with distinct scores that
    // happens after a dozen bits or so, not 32).
    uint32_t thr = 0u;
    bool exact = false;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = thr | (1u << bit);
      int c = 0;
#pragma unroll
      for (int e = 0; e < EPL; ++e) c += key[e] >= cand ? 1 : 0;
      c = wave_sum(c);
      if (c >= want) thr = cand;
      if (c == want) {  // wave-uniform
        exact = true;
        break;
      }
    }
    int need_eq;
    if (exact) {
      // every key >= thr is taken: treat them all as "equal to the threshold" takers by lowering thr's
      // role to a pure lower bound (thr - 1 is below all of them, and no other key is >= thr)
      need_eq = 0;
      thr -= 1u;  // thr >= 1 here: c == want >= 1 keys are >= cand, and cand > 0
    } else {
      int greater = 0;
#pragma unroll
      for (int e = 0; e < EPL; ++e) greater += (e * 64 + lane < nb_valid && key[e] > thr) ? 1 : 0;
      need_eq = want - wave_sum(greater);  // >= 1 by construction
    }

    int out_base = 0, eq_base = 0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const int j = e * 64 + lane;
      const bool valid = j < nb_valid;
      const bool gt = valid && key[e] > thr;
      const bool eq = valid && key[e] == thr;
      const unsigned long long eq_b = __builtin_amdgcn_ballot_w64(eq);
      const bool take = gt || (eq && eq_base + lanes_below(eq_b) < need_eq);
      const unsigned long long take_b = __builtin_amdgcn_ballot_w64(take);
      if (take) out[out_base + lanes_below(take_b)] = j;
      out_base += __popcll(take_b);
      eq_base += __popcll(eq_b);
    }
  }
  for (int s = want + lane; s < kmax; s += 64) out[s] = -1;
  if (lane == 0) cnt[row] = want;
}

template <int EPL>
hipError_t run(const float* scores, const Dims& s, int k, const int32_t* budgets, int kmax, bool force_local,
               int32_t* idx, int32_t* cnt, hipStream_t st) {
  const long long rows = s.bh() * s.nb;
  const unsigned grid = (unsigned)((rows + kRowsPerWg - 1) / kRowsPerWg);
  select_topk<EPL><<<grid, 64 * kRowsPerWg, 0, st>>>(scores, budgets, k, kmax, s.nb, s.nb_valid, rows, force_local ? 1 : 0,
                                                     idx, cnt);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_select_topk(const float* scores, const Dims& s, int k, const int32_t* budgets, int kmax,
                              bool force_local, int32_t* idx, int32_t* cnt, hipStream_t st) {
  const int epl = (s.nb + 63) / 64;
#define USV_TOPK_CASE(E) \
  if (epl <= E) return run<E>(scores, s, k, budgets, kmax, force_local, idx, cnt, st)
  USV_TOPK_CASE(1);
  USV_TOPK_CASE(2);
  USV_TOPK_CASE(4);
  USV_TOPK_CASE(8);
  USV_TOPK_CASE(12);
  USV_TOPK_CASE(16);
  USV_TOPK_CASE(20);
  USV_TOPK_CASE(24);
  USV_TOPK_CASE(32);
  USV_TOPK_CASE(48);
  USV_TOPK_CASE(64);
#undef USV_TOPK_CASE
  return hipErrorInvalidValue;  // unreachable: the API rejects nb > USV_MAX_BLOCKS
}

}  // namespace usv
