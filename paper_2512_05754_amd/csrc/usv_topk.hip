// Stage 2: per-query-block top-k key-block selection ("top-k cube selection", paper Figure 2).
//
// One 64-lane wavefront owns one score row.  The row lives in registers as the fp32 scores themselves
// (element e*64+lane in slot e).  The total order is the one of order-preserving unsigned keys
// (-0 == +0, NaN below -inf, ties towards the lower block index), but no key is ever formed per element:
// the k-th largest key is found by a bit-by-bit search over the KEY space from the most significant bit,
// and each candidate key is turned back into a float on the scalar unit, so that one pass over the row is
// one float compare per slot (the compare writes a lane mask, the scalar unit counts its bits).  Float
// compares order -0 with +0 and leave NaN out of every count, which is exactly the key order.  Passes
// whose candidate lies above the row maximum are skipped (their count is known to be 0), and the search
// stops as soon as a candidate splits off exactly k scores.  The result is a pure function of the
// (key, index) total order: bit-exact and free of atomics.  Ties at the threshold are broken towards the
// lower block index with ballot prefix counts; the survivors are written in ascending block index.
#include "usv_internal.h"

namespace usv {
namespace {

constexpr int kRowsPerWg = 4;  // 4 wavefronts, one row each

// The order-preserving key of a canonicalised fp32 with bit pattern b (never formed per element, see above):
//   NaN -> 0 (below -inf's key);  -0 -> the key of +0;  negative floats -> ~b;  the others -> b | 0x80000000.

// The float t(c) with  x >= t(c)  <=>  order_key(x) >= c  for every candidate key c >= 1:
//   c <= key(-inf): every number (NaN excluded) qualifies -> -inf;  keys of the negative floats are the
//   complemented bit patterns;  keys of the non-negative floats are the patterns with the top bit set
//   (patterns above +inf are NaNs: the compare is false for every x, and no key reaches that high).
__device__ __forceinline__ float key_threshold(uint32_t c) {
  const uint32_t num = (int32_t)c < 0 ? (c & 0x7fffffffu) : ~c;  // selects, not branches: this runs on the scalar unit
  return __uint_as_float(c <= 0x007fffffu ? 0xff800000u : num);
}

// Sum of a per-lane count over the 64 lanes, as a wave-uniform value: four DPP adds leave every 16-lane row's
// total in all of its lanes (pairs, quads, then the row rotated by 4 and by 8), and the four row totals are
// read back with v_readlane.
__device__ __forceinline__ int wave_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x124, 0xf, 0xf, false);  // row_ror:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false);  // row_ror:8
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
         __builtin_amdgcn_readlane(v, 48);
}

// Maximum of a signed integer over the 64 lanes, the same value in every lane.
__device__ __forceinline__ int wave_max_i32(int v) {
  v = max(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
  v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
  v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x124, 0xf, 0xf, false));  // row_ror:4
  v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false));  // row_ror:8
  return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
             max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

// number of set bits of `mask` below this lane
__device__ __forceinline__ int lanes_below(unsigned long long mask) {
  return __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
}

// EPL = elements per lane: row length <= 64 * EPL.  FORCE_LOCAL: every row keeps its own cube.
template <int EPL, bool FORCE_LOCAL>
__global__ __launch_bounds__(64 * kRowsPerWg) void select_topk(const float* __restrict__ scores,
                                                               const int32_t* __restrict__ budgets, int k_uniform,
                                                               int kmax, int nb, int nb_valid, long long rows,
                                                               int32_t* __restrict__ idx, int32_t* __restrict__ cnt) {
  const int lane = threadIdx.x & 63;
  // the row is the same in every lane of the wavefront: say so, and the addresses below get a scalar base
  const long long row = (long long)blockIdx.x * kRowsPerWg + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  if (row >= rows) return;  // whole wavefront leaves together; no barriers in this kernel
  const int i = (int)(row % nb);
  int32_t* out = idx + row * kmax;

  int want = budgets ? budgets[row] : k_uniform;
  want = max(0, min(want, min(kmax, nb_valid)));
  if (i >= nb_valid) want = 0;
  want = __builtin_amdgcn_readfirstlane(want);  // the same in every lane; keep the search loop scalar

  if (want > 0) {
    const float* src = scores + row * nb;
    const float kNan = __uint_as_float(0xffc00000u);  // sign bit set: see the row maximum below
    // every load of the row is in flight at once (slots past the row re-read its last score and are
    // overwritten below)
    float x[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) x[e] = src[min(e * 64 + lane, nb - 1)];
    // slots beyond the valid blocks become NaN: no compare below counts them, and the tie pass masks them
#pragma unroll
    for (int e = 0; e < EPL; ++e)
      if ((e + 1) * 64 > nb_valid) x[e] = e * 64 + lane < nb_valid ? x[e] : kNan;
    // local-cube allocation: the row's own cube is taken whatever its score, and the rest of the budget goes
    // to the best others.  It leaves the search as a NaN and re-enters at the emission.
    const bool local_lane = FORCE_LOCAL && lane == (i & 63);
    const int local_slot = FORCE_LOCAL ? (i >> 6) : -1;
    int want_s = want;
    if constexpr (FORCE_LOCAL) {
      want_s = want - 1;
#pragma unroll
      for (int e = 0; e < EPL; ++e)
        if (e == local_slot) x[e] = local_lane ? kNan : x[e];
    }

    // An upper bound of the keys present, from the maximum of the bit patterns as SIGNED integers: the
    // non-negative floats order like their patterns and lie above every pattern with the sign bit (the
    // negative floats and the NaN filler above).  A row without a positive score gets the bound key(+0);
    // a row with a (positive-pattern) NaN gets no bound.  The bound only decides which passes are skipped.
    int mi = (int)__float_as_uint(x[0]);
#pragma unroll
    for (int e = 1; e < EPL; ++e) mi = max(mi, (int)__float_as_uint(x[e]));
    mi = __builtin_amdgcn_readfirstlane(wave_max_i32(mi));
    const uint32_t key_max = mi < 0 ? 0x80000000u : (mi > 0x7f800000 ? 0xffffffffu : (0x80000000u | (uint32_t)mi));

    // thr = the want_s-th largest key.  Every candidate is >= 1, so NaNs (key 0) never count.  The search stops
    // as soon as a candidate splits off exactly want_s scores: they are the answer whatever the lower bits
    // are (with distinct scores that happens after a dozen bits or so, not 32).
    constexpr int VSLOTS = EPL >= 12 ? (EPL * 3) / 5 : 0;  // slots counted on the vector unit (see the loop)
    uint32_t thr = 0u;
    bool exact = false;
    if (want_s > 0) {
      for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = thr | (1u << bit);
        if (cand > key_max) continue;  // no key that high: the count is 0
        const float t = key_threshold(cand);
        // Count the scores >= t.  A compare writes a lane mask; its bits are counted either by the scalar unit
        // (one compare on the vector unit, a count and an add on the scalar unit) or by an add-with-carry per
        // lane and one wave-wide sum at the end (two vector instructions, none scalar).  Each unit issues one
        // instruction every four clocks per SIMD, and long rows are bound by exactly that, so they split the
        // slots between the two; short rows are latency bound and take the variant with fewer instructions.
        int c = 0;
        if constexpr (VSLOTS > 0) {
          int cl = 0;
#pragma unroll
          for (int e = 0; e < VSLOTS; ++e) cl += x[e] >= t ? 1 : 0;
          c = wave_sum(cl);
        }
#pragma unroll
        for (int e = VSLOTS; e < EPL; ++e) c += __popcll(__builtin_amdgcn_ballot_w64(x[e] >= t));
        if (c < want_s) continue;
        thr = cand;
        if (c == want_s) {
          exact = true;
          break;
        }
      }
    }
    // Exact: every score >= t(thr) is taken.  (want_s == 0, nothing but the local cube: "x >= NaN" takes no one.)
    // Not exact: thr is the key of the want_s-th largest score and more than want_s scores are >= it.  The ones
    // above it are all taken, the ones equal to it in ascending block index until the budget is full.
    // thr == 0: the numbers ran out, and the NaNs of the valid blocks are the equals.
    float above = want_s == 0 ? kNan : key_threshold(exact ? thr : thr + 1u);  // thr <= key(+inf): no overflow
    int need_eq = 0;
    float from = kNan;
    if (want_s > 0 && !exact) {
      from = key_threshold(thr);
      int greater = 0;
#pragma unroll
      for (int e = 0; e < EPL; ++e) greater += __popcll(__builtin_amdgcn_ballot_w64(x[e] >= above));
      need_eq = want_s - greater;  // >= 1 by construction
    }
    if (need_eq == 0) {
      int out_base = 0;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        bool take = x[e] >= above;
        if constexpr (FORCE_LOCAL) take = take || (e == local_slot && local_lane);
        const unsigned long long take_b = __builtin_amdgcn_ballot_w64(take);
        if (take) out[out_base + lanes_below(take_b)] = e * 64 + lane;
        out_base += __popcll(take_b);
      }
    } else {
      int out_base = 0, eq_base = 0;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const int j = e * 64 + lane;
        const bool is_local = FORCE_LOCAL && e == local_slot && local_lane;
        const bool gt = x[e] >= above;
        const bool ge = thr == 0u ? (j < nb_valid && !is_local) : x[e] >= from;
        const bool eq = ge && !gt;
        const unsigned long long eq_b = __builtin_amdgcn_ballot_w64(eq);
        const bool take = gt || is_local || (eq && eq_base + lanes_below(eq_b) < need_eq);
        const unsigned long long take_b = __builtin_amdgcn_ballot_w64(take);
        if (take) out[out_base + lanes_below(take_b)] = j;
        out_base += __popcll(take_b);
        eq_base += __popcll(eq_b);
      }
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
  if (force_local)
    select_topk<EPL, true><<<grid, 64 * kRowsPerWg, 0, st>>>(scores, budgets, k, kmax, s.nb, s.nb_valid, rows, idx, cnt);
  else
    select_topk<EPL, false><<<grid, 64 * kRowsPerWg, 0, st>>>(scores, budgets, k, kmax, s.nb, s.nb_valid, rows, idx, cnt);
  return hipGetLastError();
}

// Work order of the attention launch: per (batch, head) the query blocks sorted by
//   (list length descending, where the list lies ascending, block index ascending),
// "where the list lies" being the entries at 1/4, 1/2 and 3/4 of the list, each reduced to one of 64 buckets
// of the block range and compared lexicographically.  Workgroups that run together then have lists of similar
// length and similar placement: their ascending sweeps over the head's K/V stay together in the XCD's L2, and
// the last round of the launch is made of the shortest lists.  One workgroup per (batch, head): the keys,
// packed with the block index into 64 bits (all distinct, so the result is deterministic), are sorted in LDS
// with a bitonic network.
constexpr int kOrderThreads = 1024;

__global__ __launch_bounds__(kOrderThreads) void attn_work_order(const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt,
                                                                 int32_t* __restrict__ order, int nb, int kmax, int n2) {
  extern __shared__ unsigned long long keys[];  // n2 = nb rounded up to a power of two
  const int tid = threadIdx.x;
  const long long row0 = (long long)blockIdx.x * nb;
  for (int i = tid; i < n2; i += kOrderThreads) {
    unsigned long long key = ~0ull;  // padding sorts last
    if (i < nb) {
      const int c = min(max(cnt[row0 + i], 0), kmax);
      unsigned pos = 0u;
      if (idx && c > 0) {
        const int32_t* list = idx + (row0 + i) * kmax;
#pragma unroll
        for (int quarter = 1; quarter <= 3; ++quarter) {
          const int j = min(max(list[(c - 1) * quarter / 4], 0), nb - 1);
          pos = (pos << 6) | (unsigned)((long long)j * 64 / nb);
        }
      }
      key = ((unsigned long long)(kmax - c) << 30) | ((unsigned long long)pos << 12) | (unsigned)i;
    }
    keys[i] = key;
  }
  __syncthreads();
  for (int k = 2; k <= n2; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < n2 / 2; t += kOrderThreads) {
        const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1));  // the lower index of pair t at distance j
        const int hi = lo | j;
        const unsigned long long a = keys[lo], b = keys[hi];
        const bool up = (lo & k) == 0;
        if ((a > b) == up) {
          keys[lo] = b;
          keys[hi] = a;
        }
      }
      __syncthreads();
    }
  }
  for (int s = tid; s < nb; s += kOrderThreads) order[row0 + s] = (int32_t)(keys[s] & 0xfffu);
}

}  // namespace

hipError_t launch_attn_work_order(const int32_t* idx, const int32_t* cnt, const Dims& s, int kmax, int32_t* work_order,
                                  hipStream_t st) {
  int n2 = 2;
  while (n2 < s.nb) n2 <<= 1;  // <= 4096: 32 KiB of LDS
  attn_work_order<<<(unsigned)s.bh(), kOrderThreads, (size_t)n2 * sizeof(unsigned long long), st>>>(idx, cnt, work_order, s.nb,
                                                                                                      kmax, n2);
  return hipGetLastError();
}

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
