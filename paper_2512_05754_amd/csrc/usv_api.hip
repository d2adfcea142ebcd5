// C ABI of libusv: host-side argument validation and dispatch to the HIP kernels.
// All checks run before anything is launched, so the error paths need no GPU.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>

#include "usv_internal.h"

namespace {

thread_local char g_err[256] = "";

usv_status fail(usv_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks the shape fields the three stages share and fills Dims.
usv_status check_shape(const usv_shape* sh, bool need_dtype, usv::Dims* out) {
  if (!sh) return fail(USV_ERR_INVALID_ARG, "shape is NULL");
  if (sh->batch < 1 || sh->heads < 1) return fail(USV_ERR_INVALID_ARG, "batch and heads must be >= 1");
  if (sh->block != usv::kBlock) return fail(USV_ERR_UNSUPPORTED, "block must be 64 (got %d)", sh->block);
  if (sh->seq_len < sh->block || sh->seq_len % sh->block != 0)
    return fail(USV_ERR_INVALID_ARG, "seq_len (%d) must be a positive multiple of block", sh->seq_len);
  if (sh->seq_valid < 1 || sh->seq_valid > sh->seq_len)
    return fail(USV_ERR_INVALID_ARG, "seq_valid (%d) must be in [1, seq_len]", sh->seq_valid);
  const int nb = sh->seq_len / sh->block;
  if (nb > USV_MAX_BLOCKS) return fail(USV_ERR_UNSUPPORTED, "more than %d blocks (got %d)", USV_MAX_BLOCKS, nb);
  if ((long long)sh->batch * sh->heads > 65535) return fail(USV_ERR_UNSUPPORTED, "batch * heads must be <= 65535");
  if ((long long)sh->batch * sh->heads * nb > 0x7fffffffLL / 8)
    return fail(USV_ERR_UNSUPPORTED, "batch * heads * blocks too large");
  if (need_dtype) {
    if (sh->head_dim != 64 && sh->head_dim != 128)
      return fail(USV_ERR_UNSUPPORTED, "head_dim must be 64 or 128 (got %d)", sh->head_dim);
    if (sh->dtype != USV_F32 && sh->dtype != USV_BF16)
      return fail(USV_ERR_UNSUPPORTED, "dtype must be USV_F32 or USV_BF16 (got %d)", sh->dtype);
  }
  out->B = sh->batch;
  out->Hh = sh->heads;
  out->N = sh->seq_len;
  out->Nv = sh->seq_valid;
  out->d = sh->head_dim;
  out->nb = nb;
  out->nb_valid = (sh->seq_valid + sh->block - 1) / sh->block;
  out->bf16 = sh->dtype == USV_BF16;
  return USV_OK;
}

usv_status check_ptr(const void* p, const char* name) {
  if (!p) return fail(USV_ERR_INVALID_ARG, "%s is NULL", name);
  if (!aligned16(p)) return fail(USV_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
  return USV_OK;
}

usv_status hip_result(hipError_t e, const char* what) {
  if (e == hipSuccess) {
    g_err[0] = '\0';
    return USV_OK;
  }
  return fail(USV_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// Checks the grid against the shape and fills CubeGrid.
usv_status check_grid(const usv_grid* g, const usv_shape* sh, usv::CubeGrid* out) {
  if (!g) return fail(USV_ERR_INVALID_ARG, "grid is NULL");
  if (g->T < 1 || g->H < 1 || g->W < 1) return fail(USV_ERR_INVALID_ARG, "grid extents must be >= 1");
  if (g->ct < 1 || g->ch < 1 || g->cw < 1) return fail(USV_ERR_INVALID_ARG, "cube extents must be >= 1");
  if ((long long)g->ct * g->ch * g->cw != usv::kBlock)
    return fail(USV_ERR_UNSUPPORTED, "cube must hold 64 tokens (got %d x %d x %d)", g->ct, g->ch, g->cw);
  const long long tokens = (long long)g->T * g->H * g->W;
  if (tokens > (long long)USV_MAX_BLOCKS * usv::kBlock)
    return fail(USV_ERR_UNSUPPORTED, "grid holds more than %d tokens", USV_MAX_BLOCKS * usv::kBlock);
  if (sh && tokens != sh->seq_valid)
    return fail(USV_ERR_INVALID_ARG, "grid holds %lld tokens but seq_valid is %d", tokens, sh->seq_valid);
  *out = usv::CubeGrid{g->T, g->H, g->W, g->ct, g->ch, g->cw, g->T / g->ct, g->H / g->ch, g->W / g->cw};
  return USV_OK;
}

// Raster strides in bytes (contiguous [B, Hh, Nv, d] when `st` is NULL), checked for 16-byte rows that do not overlap.
usv_status check_strides(const usv_strides* st, const usv::Dims& s, long long out_bytes[3], long long esz = 0) {
  if (esz == 0) esz = s.bf16 ? 2 : 4;
  long long e[3] = {(long long)s.Hh * s.Nv * s.d, (long long)s.Nv * s.d, (long long)s.d};
  if (st) {
    e[0] = st->batch;
    e[1] = st->head;
    e[2] = st->token;
  }
  for (int i = 0; i < 3; ++i) {
    if (e[i] < 0 || e[i] > (1LL << 40)) return fail(USV_ERR_INVALID_ARG, "raster strides must be in [0, 2^40] elements");
    if ((e[i] * esz) % 16 != 0) return fail(USV_ERR_INVALID_ARG, "raster strides must be multiples of 16 bytes");
    out_bytes[i] = e[i] * esz;
  }
  if (e[2] < s.d) return fail(USV_ERR_INVALID_ARG, "token stride (%lld) is smaller than head_dim: rows overlap", e[2]);
  if (s.Hh > 1 && e[1] < s.d) return fail(USV_ERR_INVALID_ARG, "head stride (%lld) is smaller than head_dim: rows overlap", e[1]);
  if (s.B > 1 && e[0] < s.d) return fail(USV_ERR_INVALID_ARG, "batch stride (%lld) is smaller than head_dim: rows overlap", e[0]);
  return USV_OK;
}

// Token merging: `sh` describes the merged tensors, `g` the raster grid and the merge block.
// Fills Dims, MergeGrid, the raster token count N and r = N - seq_valid (sources to merge).
usv_status check_merge(const usv_shape* sh, const usv_grid* g, usv::Dims* s, usv::MergeGrid* mg, int* N, int* r) {
  const usv_status st = check_shape(sh, true, s);
  if (st != USV_OK) return st;
  if (!g) return fail(USV_ERR_INVALID_ARG, "grid is NULL");
  if (g->T < 1 || g->H < 1 || g->W < 1) return fail(USV_ERR_INVALID_ARG, "grid extents must be >= 1");
  if (g->ct < 1 || g->ch < 1 || g->cw < 1) return fail(USV_ERR_INVALID_ARG, "merge block extents must be >= 1");
  const long long tokens = (long long)g->T * g->H * g->W;
  if (tokens > (long long)USV_MAX_BLOCKS * usv::kBlock)
    return fail(USV_ERR_UNSUPPORTED, "grid holds more than %d tokens", USV_MAX_BLOCKS * usv::kBlock);
  *mg = usv::MergeGrid{g->T, g->H, g->W, g->ct, g->ch, g->cw, (g->T + g->ct - 1) / g->ct, (g->H + g->ch - 1) / g->ch,
                       (g->W + g->cw - 1) / g->cw};
  const long long n_dst = (long long)mg->nT * mg->nH * mg->nW;
  if (sh->seq_valid > tokens || sh->seq_valid < n_dst)
    return fail(USV_ERR_INVALID_ARG, "seq_valid (%d merged rows) must lie between the %lld destinations and the %lld tokens of the grid",
                sh->seq_valid, n_dst, tokens);
  *N = (int)tokens;
  *r = (int)(tokens - sh->seq_valid);
  return USV_OK;
}

#define USV_TRY(expr)                    \
  do {                                   \
    const usv_status st__ = (expr);      \
    if (st__ != USV_OK) return st__;     \
  } while (0)

}  // namespace

extern "C" {

size_t usv_workspace_bytes(const usv_shape* shape) {
  usv::Dims s;
  if (check_shape(shape, true, &s) != USV_OK) return 0;
  return (size_t)2 * s.bh() * s.nb * s.d * sizeof(float);
}

usv_status usv_block_scores(const void* q, const void* k, const usv_shape* shape, float* scores, void* ws,
                            size_t ws_bytes, void* stream) {
  usv::Dims s;
  USV_TRY(check_shape(shape, true, &s));
  USV_TRY(check_ptr(q, "q"));
  USV_TRY(check_ptr(k, "k"));
  USV_TRY(check_ptr(scores, "scores"));
  const size_t need = usv_workspace_bytes(shape);
  if (!ws || !aligned16(ws) || ws_bytes < need)
    return fail(USV_ERR_WORKSPACE, "workspace needs %zu bytes, 16-byte aligned (got %zu)", need, ws_bytes);
  return hip_result(usv::launch_block_scores(q, k, s, scores, static_cast<float*>(ws), static_cast<hipStream_t>(stream)),
                    "usv_block_scores launch");
}

// ---- stage 1 for callers that cannot allocate: the pooled means live in a static device array ----------
namespace {

// Each GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
// In host code the name is only a handle for hipGetSymbolAddress: the per-device address it returns is what
// kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[USV_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, resolved on first use

usv_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(USV_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(USV_ERR_UNSUPPORTED, "device ordinal %d is beyond %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // the current device's copy
    if (e != hipSuccess || !p) return fail(USV_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return USV_OK;
}

}  // namespace

usv_status usv_block_scores_static(const void* q, const void* k, const usv_shape* shape, float* scores, void* stream) {
  usv::Dims s;
  USV_TRY(check_shape(shape, true, &s));
  USV_TRY(check_ptr(q, "q"));
  USV_TRY(check_ptr(k, "k"));
  USV_TRY(check_ptr(scores, "scores"));
  const size_t need = usv_workspace_bytes(shape);
  if (need > (size_t)USV_STATIC_SCRATCH_BYTES)
    return fail(USV_ERR_WORKSPACE, "the pooled means of this shape need %zu bytes, the static scratch holds %zu: use usv_block_scores",
                need, (size_t)USV_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  USV_TRY(static_scratch(&ws));
  // every element of the scratch that the product kernel reads is written by the pooling kernel of this
  // same call first (same stream), so nothing needs clearing between calls
  return hip_result(usv::launch_block_scores(q, k, s, scores, static_cast<float*>(ws), static_cast<hipStream_t>(stream)),
                    "usv_block_scores_static launch");
}

usv_status usv_select_topk(const float* scores, const usv_shape* shape, int32_t k, const int32_t* budgets,
                           int32_t kmax, int32_t* idx, int32_t* cnt, void* stream) {
  return usv_select_topk_ex(scores, shape, k, budgets, kmax, 0u, idx, cnt, stream);
}

usv_status usv_select_topk_ex(const float* scores, const usv_shape* shape, int32_t k, const int32_t* budgets,
                              int32_t kmax, uint32_t flags, int32_t* idx, int32_t* cnt, void* stream) {
  usv::Dims s;
  if (flags & ~(uint32_t)USV_TOPK_FORCE_LOCAL) return fail(USV_ERR_INVALID_ARG, "unknown flag bits 0x%x", flags);
  USV_TRY(check_shape(shape, false, &s));
  USV_TRY(check_ptr(scores, "scores"));
  USV_TRY(check_ptr(idx, "idx"));
  USV_TRY(check_ptr(cnt, "cnt"));
  if (kmax < 1 || kmax > s.nb) return fail(USV_ERR_INVALID_ARG, "kmax (%d) must be in [1, blocks = %d]", kmax, s.nb);
  if (budgets) {
    USV_TRY(check_ptr(budgets, "budgets"));
  } else if (k < 1 || k > kmax) {
    return fail(USV_ERR_INVALID_ARG, "k (%d) must be in [1, kmax = %d]", k, kmax);
  }
  return hip_result(usv::launch_select_topk(scores, s, k, budgets, kmax, (flags & USV_TOPK_FORCE_LOCAL) != 0, idx, cnt,
                                            static_cast<hipStream_t>(stream)),
                    "usv_select_topk launch");
}

usv_status usv_block_sparse_attn(const void* q, const void* k, const void* v, const usv_shape* shape,
                                 const int32_t* idx, const int32_t* cnt, int32_t kmax, float scale,
                                 int32_t out_dtype, void* out, float* lse, void* stream) {
  return usv_block_sparse_attn_fused(q, k, v, shape, idx, cnt, kmax, scale, nullptr, nullptr, nullptr, out_dtype, out,
                                     lse, stream);
}

usv_status usv_attn_work_order(const int32_t* idx, const int32_t* cnt, const usv_shape* shape, int32_t kmax,
                               int32_t* work_order, void* stream) {
  usv::Dims s;
  USV_TRY(check_shape(shape, false, &s));
  if (idx) USV_TRY(check_ptr(idx, "idx"));
  USV_TRY(check_ptr(cnt, "cnt"));
  USV_TRY(check_ptr(work_order, "work_order"));
  if (kmax < 1 || kmax > s.nb) return fail(USV_ERR_INVALID_ARG, "kmax (%d) must be in [1, blocks = %d]", kmax, s.nb);
  return hip_result(usv::launch_attn_work_order(idx, cnt, s, kmax, work_order, static_cast<hipStream_t>(stream)),
                    "usv_attn_work_order launch");
}

namespace {
usv_status attn_any(const void* q, const void* k, const void* v, const usv_shape* shape, const int32_t* idx,
                    const int32_t* cnt, int32_t kmax, const int32_t* work_order, float scale, const float* coarse,
                    const void* gate_fine, const void* gate_coarse, int32_t out_dtype, void* out, float* lse, void* stream);
}

usv_status usv_block_sparse_attn_ordered(const void* q, const void* k, const void* v, const usv_shape* shape,
                                         const int32_t* idx, const int32_t* cnt, int32_t kmax, const int32_t* work_order,
                                         float scale, int32_t out_dtype, void* out, float* lse, void* stream) {
  if (work_order) USV_TRY(check_ptr(work_order, "work_order"));
  return attn_any(q, k, v, shape, idx, cnt, kmax, work_order, scale, nullptr, nullptr, nullptr, out_dtype, out, lse, stream);
}

usv_status usv_block_sparse_attn_fused(const void* q, const void* k, const void* v, const usv_shape* shape,
                                       const int32_t* idx, const int32_t* cnt, int32_t kmax, float scale,
                                       const float* coarse, const void* gate_fine, const void* gate_coarse,
                                       int32_t out_dtype, void* out, float* lse, void* stream) {
  return attn_any(q, k, v, shape, idx, cnt, kmax, nullptr, scale, coarse, gate_fine, gate_coarse, out_dtype, out, lse, stream);
}

namespace {
usv_status attn_any(const void* q, const void* k, const void* v, const usv_shape* shape, const int32_t* idx,
                    const int32_t* cnt, int32_t kmax, const int32_t* work_order, float scale, const float* coarse,
                    const void* gate_fine, const void* gate_coarse, int32_t out_dtype, void* out, float* lse, void* stream) {
  usv::Dims s;
  USV_TRY(check_shape(shape, true, &s));
  USV_TRY(check_ptr(q, "q"));
  USV_TRY(check_ptr(k, "k"));
  USV_TRY(check_ptr(v, "v"));
  USV_TRY(check_ptr(idx, "idx"));
  USV_TRY(check_ptr(cnt, "cnt"));
  USV_TRY(check_ptr(out, "out"));
  if (lse && !aligned16(lse)) return fail(USV_ERR_INVALID_ARG, "lse is not 16-byte aligned");
  if (kmax < 1 || kmax > s.nb) return fail(USV_ERR_INVALID_ARG, "kmax (%d) must be in [1, blocks = %d]", kmax, s.nb);
  if (out_dtype != shape->dtype && !(s.bf16 && out_dtype == USV_F32))
    return fail(USV_ERR_UNSUPPORTED, "out_dtype must equal the input dtype, or be USV_F32 for bf16 inputs");
  if (std::isnan(scale) || std::isinf(scale)) return fail(USV_ERR_INVALID_ARG, "scale must be finite");
  if (!coarse && (gate_fine || gate_coarse)) return fail(USV_ERR_INVALID_ARG, "gates without coarse");
  if (coarse && !aligned16(coarse)) return fail(USV_ERR_INVALID_ARG, "coarse is not 16-byte aligned");
  if (gate_fine && !aligned16(gate_fine)) return fail(USV_ERR_INVALID_ARG, "gate_fine is not 16-byte aligned");
  if (gate_coarse && !aligned16(gate_coarse)) return fail(USV_ERR_INVALID_ARG, "gate_coarse is not 16-byte aligned");
  if (scale <= 0.f) scale = 1.0f / std::sqrt((float)s.d);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (s.bf16) {
    const usv::FuseArgs fuse{coarse, static_cast<const uint16_t*>(gate_fine), static_cast<const uint16_t*>(gate_coarse)};
    return hip_result(usv::launch_attn_bf16(q, k, v, s, idx, cnt, kmax, scale, out, out_dtype == USV_F32, lse, fuse, st,
                                            work_order),
                      "usv_block_sparse_attn launch");
  }
  // fp32 inputs (the accuracy path; it takes the query blocks in index order whatever work_order says): attention,
  // then the fusion kernel in place
  hipError_t e = usv::launch_attn_f32(static_cast<const float*>(q), static_cast<const float*>(k),
                                      static_cast<const float*>(v), s, idx, cnt, kmax, scale, static_cast<float*>(out),
                                      lse, st);
  if (e == hipSuccess && coarse)
    e = usv::launch_fuse_outputs(out, true, coarse, gate_fine, gate_coarse, true, out, true, s, st);
  return hip_result(e, "usv_block_sparse_attn launch");
}
}  // namespace

size_t usv_coarse_workspace_bytes(const usv_shape* shape) {
  usv::Dims s;
  if (check_shape(shape, true, &s) != USV_OK) return 0;
  return (size_t)s.bh() * s.nb * s.d * sizeof(float);
}

usv_status usv_coarse_attn(const float* scores, const void* v, const usv_shape* shape, float* coarse, void* ws,
                           size_t ws_bytes, void* stream) {
  usv::Dims s;
  USV_TRY(check_shape(shape, true, &s));
  USV_TRY(check_ptr(scores, "scores"));
  USV_TRY(check_ptr(v, "v"));
  USV_TRY(check_ptr(coarse, "coarse"));
  const size_t need = usv_coarse_workspace_bytes(shape);
  if (!ws || !aligned16(ws) || ws_bytes < need)
    return fail(USV_ERR_WORKSPACE, "workspace needs %zu bytes, 16-byte aligned (got %zu)", need, ws_bytes);
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = usv::launch_pool_means(v, s, static_cast<float*>(ws), st);
  if (e == hipSuccess) e = usv::launch_coarse_attn(scores, static_cast<const float*>(ws), s, coarse, st);
  return hip_result(e, "usv_coarse_attn launch");
}

usv_status usv_fuse_outputs(const void* fine, int32_t fine_dtype, const float* coarse, const void* gate_fine,
                            const void* gate_coarse, const usv_shape* shape, int32_t out_dtype, void* out,
                            void* stream) {
  usv::Dims s;
  USV_TRY(check_shape(shape, true, &s));
  USV_TRY(check_ptr(fine, "fine"));
  USV_TRY(check_ptr(coarse, "coarse"));
  USV_TRY(check_ptr(out, "out"));
  if (gate_fine && !aligned16(gate_fine)) return fail(USV_ERR_INVALID_ARG, "gate_fine is not 16-byte aligned");
  if (gate_coarse && !aligned16(gate_coarse)) return fail(USV_ERR_INVALID_ARG, "gate_coarse is not 16-byte aligned");
  if ((fine_dtype != USV_F32 && fine_dtype != USV_BF16) || (out_dtype != USV_F32 && out_dtype != USV_BF16))
    return fail(USV_ERR_UNSUPPORTED, "fine_dtype and out_dtype must be USV_F32 or USV_BF16");
  if (out == fine && out_dtype != fine_dtype)
    return fail(USV_ERR_INVALID_ARG, "in-place fusion (out == fine) needs out_dtype == fine_dtype");
  return hip_result(usv::launch_fuse_outputs(fine, fine_dtype == USV_F32, coarse, gate_fine, gate_coarse, !s.bf16, out,
                                             out_dtype == USV_F32, s, static_cast<hipStream_t>(stream)),
                    "usv_fuse_outputs launch");
}

size_t usv_entropy_workspace_bytes(const usv_shape* shape) {
  usv::Dims s;
  if (check_shape(shape, false, &s) != USV_OK) return 0;
  return (size_t)s.bh() * ((s.nb_valid + 31) / 32) * s.nb * sizeof(float);
}

usv_status usv_attn_entropy(const float* scores, const usv_shape* shape, float* entropy, void* ws, size_t ws_bytes,
                            void* stream) {
  usv::Dims s;
  USV_TRY(check_shape(shape, false, &s));
  USV_TRY(check_ptr(scores, "scores"));
  if (!entropy) return fail(USV_ERR_INVALID_ARG, "entropy is NULL");
  if (reinterpret_cast<uintptr_t>(entropy) & 3u) return fail(USV_ERR_INVALID_ARG, "entropy is not 4-byte aligned");
  const size_t need = usv_entropy_workspace_bytes(shape);
  if (!ws || !aligned16(ws) || ws_bytes < need)
    return fail(USV_ERR_WORKSPACE, "workspace needs %zu bytes, 16-byte aligned (got %zu)", need, ws_bytes);
  return hip_result(usv::launch_attn_entropy(scores, s, entropy, static_cast<float*>(ws), static_cast<hipStream_t>(stream)),
                    "usv_attn_entropy launch");
}

usv_status usv_entropy_allocate(const float* entropy, int32_t layers, float rho_bar, float gamma, float rho_min,
                                float rho_max, float* rho) {
  if (!entropy || !rho) return fail(USV_ERR_INVALID_ARG, "entropy or rho is NULL");
  if (layers < 1) return fail(USV_ERR_INVALID_ARG, "layers must be >= 1");
  if (!(gamma >= 1.0f)) return fail(USV_ERR_INVALID_ARG, "gamma must be >= 1");
  if (!(rho_min <= rho_max)) return fail(USV_ERR_INVALID_ARG, "rho_min must be <= rho_max");
  double mean = 0.0;
  for (int l = 0; l < layers; ++l) {
    if (!(entropy[l] >= 0.0f && entropy[l] <= 1.0f + 1e-6f))
      return fail(USV_ERR_INVALID_ARG, "entropy[%d] = %g is outside [0, 1]", l, (double)entropy[l]);
    mean += std::pow(std::fmax(0.0, 1.0 - (double)entropy[l]), (double)gamma);
  }
  mean /= layers;
  for (int l = 0; l < layers; ++l) {
    const double w = std::pow(std::fmax(0.0, 1.0 - (double)entropy[l]), (double)gamma);
    // every layer at entropy 1 carries no weight at all: keep the base schedule
    const double r = mean > 0.0 ? (double)rho_bar * w / mean : (double)rho_bar;
    rho[l] = (float)std::fmin(std::fmax(r, (double)rho_min), (double)rho_max);
  }
  g_err[0] = '\0';
  return USV_OK;
}

size_t usv_merge_workspace_bytes(const usv_shape* shape, const usv_grid* grid) {
  usv::Dims s;
  usv::MergeGrid g;
  int N, r;
  if (check_merge(shape, grid, &s, &g, &N, &r) != USV_OK) return 0;
  return (size_t)s.B * N * (s.d + 1) * sizeof(float);
}

usv_status usv_merge_similarity(const void* k, const usv_shape* shape, const usv_grid* grid, float* u, int32_t* blk,
                                void* ws, size_t ws_bytes, void* stream) {
  usv::Dims s;
  usv::MergeGrid g;
  int N, r;
  USV_TRY(check_merge(shape, grid, &s, &g, &N, &r));
  USV_TRY(check_ptr(k, "k"));
  USV_TRY(check_ptr(u, "u"));
  USV_TRY(check_ptr(blk, "blk"));
  const size_t need = usv_merge_workspace_bytes(shape, grid);
  if (!ws || !aligned16(ws) || ws_bytes < need)
    return fail(USV_ERR_WORKSPACE, "workspace needs %zu bytes, 16-byte aligned (got %zu)", need, ws_bytes);
  return hip_result(usv::launch_merge_similarity(k, s, g, N, u, blk, static_cast<float*>(ws), static_cast<hipStream_t>(stream)),
                    "usv_merge_similarity launch");
}

size_t usv_merge_plan_workspace_bytes(const usv_shape* shape, const usv_grid* grid) {
  usv::Dims s;
  usv::MergeGrid g;
  int N, r;
  if (check_merge(shape, grid, &s, &g, &N, &r) != USV_OK) return 0;
  return usv::merge_plan_workspace_bytes(s.B, N);
}

usv_status usv_merge_plan(const float* u, const int32_t* blk, const usv_shape* shape, const usv_grid* grid,
                          int32_t* row_of, int32_t* src_of, void* ws, size_t ws_bytes, void* stream) {
  usv::Dims s;
  usv::MergeGrid g;
  int N, r;
  USV_TRY(check_merge(shape, grid, &s, &g, &N, &r));
  USV_TRY(check_ptr(u, "u"));
  USV_TRY(check_ptr(blk, "blk"));
  USV_TRY(check_ptr(row_of, "row_of"));
  USV_TRY(check_ptr(src_of, "src_of"));
  if (ws) {
    const size_t need = usv::merge_plan_workspace_bytes(s.B, N);
    if (!aligned16(ws) || ws_bytes < need)
      return fail(USV_ERR_WORKSPACE, "workspace needs %zu bytes, 16-byte aligned (got %zu)", need, ws_bytes);
  }
  return hip_result(usv::launch_merge_select(u, blk, g, s.B, N, r, row_of, src_of, ws, static_cast<hipStream_t>(stream)),
                    "usv_merge_plan launch");
}

usv_status usv_merge_apply(const void* x, const usv_shape* shape, const usv_grid* grid, const int32_t* row_of,
                           const int32_t* src_of, void* out, void* stream) {
  usv::Dims s;
  usv::MergeGrid g;
  int N, r;
  USV_TRY(check_merge(shape, grid, &s, &g, &N, &r));
  USV_TRY(check_ptr(x, "x"));
  USV_TRY(check_ptr(row_of, "row_of"));
  USV_TRY(check_ptr(src_of, "src_of"));
  USV_TRY(check_ptr(out, "out"));
  return hip_result(usv::launch_merge_rows(x, s, g, N, row_of, src_of, out, static_cast<hipStream_t>(stream)),
                    "usv_merge_apply launch");
}

usv_status usv_unmerge_apply(const void* y, const usv_shape* shape, const usv_grid* grid, const int32_t* row_of,
                             void* out, void* stream) {
  usv::Dims s;
  usv::MergeGrid g;
  int N, r;
  USV_TRY(check_merge(shape, grid, &s, &g, &N, &r));
  USV_TRY(check_ptr(y, "y"));
  USV_TRY(check_ptr(row_of, "row_of"));
  USV_TRY(check_ptr(out, "out"));
  return hip_result(usv::launch_unmerge_rows(y, s, N, row_of, out, static_cast<hipStream_t>(stream)),
                    "usv_unmerge_apply launch");
}

// Fills RasterArgs from a usv_raster view (strides in elements -> bytes).
usv_status check_raster(const usv_raster* view, const usv::Dims& s, long long out_esz, usv::RasterArgs* ras) {
  if (!view) return fail(USV_ERR_INVALID_ARG, "raster view is NULL");
  USV_TRY(check_ptr(view->order, "order"));
  long long in_b[3], out_b[3];
  USV_TRY(check_strides(view->in_strides.token ? &view->in_strides : nullptr, s, in_b));
  USV_TRY(check_strides(view->out_strides.token ? &view->out_strides : nullptr, s, out_b, out_esz));
  // the tile requests carry the row offset in 32 bits
  if ((long long)s.Nv * in_b[2] > 0x7fffffffLL - 65536)
    return fail(USV_ERR_UNSUPPORTED, "seq_valid * token stride must stay below 2 GiB");
  if (view->block_valid) USV_TRY(check_ptr(view->block_valid, "block_valid"));
  *ras = usv::RasterArgs{view->order, in_b[2], in_b[1], in_b[0], out_b[2], out_b[1], out_b[0], s.Hh, view->block_valid};
  return USV_OK;
}

// One cube per block: every block holds a token, whatever seq_valid (the raster token count) would leave of it.
void all_blocks_live(const usv_raster* view, usv::Dims* s) {
  if (view->block_valid) s->nb_valid = s->nb;
}

int32_t usv_cube_count(const usv_grid* grid) {
  usv::CubeGrid g;
  if (check_grid(grid, nullptr, &g) != USV_OK) return 0;
  const long long n = (long long)((g.T + g.ct - 1) / g.ct) * ((g.H + g.ch - 1) / g.ch) * ((g.W + g.cw - 1) / g.cw);
  return n > USV_MAX_BLOCKS ? 0 : (int32_t)n;
}

usv_status usv_cube_order_padded(const usv_grid* grid, int32_t* order, int32_t* block_valid, void* stream) {
  usv::CubeGrid g;
  USV_TRY(check_grid(grid, nullptr, &g));
  USV_TRY(check_ptr(order, "order"));
  USV_TRY(check_ptr(block_valid, "block_valid"));
  if (usv_cube_count(grid) == 0) return fail(USV_ERR_UNSUPPORTED, "more than %d cubes", USV_MAX_BLOCKS);
  return hip_result(usv::launch_cube_order_padded(order, block_valid, g, static_cast<hipStream_t>(stream)),
                    "usv_cube_order_padded launch");
}

usv_status usv_cube_order(const usv_shape* shape, const usv_grid* grid, int32_t* order, void* stream) {
  usv::Dims s;
  usv::CubeGrid g;
  USV_TRY(check_shape(shape, false, &s));
  USV_TRY(check_grid(grid, shape, &g));
  USV_TRY(check_ptr(order, "order"));
  return hip_result(usv::launch_cube_order(order, g, s.N, s.Nv, static_cast<hipStream_t>(stream)), "usv_cube_order launch");
}

usv_status usv_block_scores_raster(const void* q, const void* k, const usv_shape* shape, const usv_raster* view,
                                   float* scores, void* ws, size_t ws_bytes, void* stream) {
  usv::Dims s;
  usv::RasterArgs ras;
  USV_TRY(check_shape(shape, true, &s));
  USV_TRY(check_raster(view, s, s.bf16 ? 2 : 4, &ras));
  all_blocks_live(view, &s);
  USV_TRY(check_ptr(q, "q"));
  USV_TRY(check_ptr(k, "k"));
  USV_TRY(check_ptr(scores, "scores"));
  const size_t need = usv_workspace_bytes(shape);
  if (!ws || !aligned16(ws) || ws_bytes < need)
    return fail(USV_ERR_WORKSPACE, "workspace needs %zu bytes, 16-byte aligned (got %zu)", need, ws_bytes);
  return hip_result(usv::launch_block_scores(q, k, s, scores, static_cast<float*>(ws), static_cast<hipStream_t>(stream), &ras),
                    "usv_block_scores_raster launch");
}

usv_status usv_block_sparse_attn_raster(const void* q, const void* k, const void* v, const usv_shape* shape,
                                        const usv_raster* view, const int32_t* idx, const int32_t* cnt, int32_t kmax,
                                        float scale, int32_t out_dtype, void* out, float* lse, void* stream) {
  return usv_block_sparse_attn_raster_fused(q, k, v, shape, view, idx, cnt, kmax, scale, nullptr, nullptr, nullptr,
                                            out_dtype, out, lse, stream);
}

usv_status usv_coarse_attn_raster(const float* scores, const void* v, const usv_shape* shape, const usv_raster* view,
                                  float* coarse, void* ws, size_t ws_bytes, void* stream) {
  usv::Dims s;
  usv::RasterArgs ras;
  USV_TRY(check_shape(shape, true, &s));
  USV_TRY(check_raster(view, s, s.bf16 ? 2 : 4, &ras));
  all_blocks_live(view, &s);
  USV_TRY(check_ptr(scores, "scores"));
  USV_TRY(check_ptr(v, "v"));
  USV_TRY(check_ptr(coarse, "coarse"));
  const size_t need = usv_coarse_workspace_bytes(shape);
  if (!ws || !aligned16(ws) || ws_bytes < need)
    return fail(USV_ERR_WORKSPACE, "workspace needs %zu bytes, 16-byte aligned (got %zu)", need, ws_bytes);
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = usv::launch_pool_means(v, s, static_cast<float*>(ws), st, &ras);
  if (e == hipSuccess) e = usv::launch_coarse_attn(scores, static_cast<const float*>(ws), s, coarse, st);
  return hip_result(e, "usv_coarse_attn_raster launch");
}

usv_status usv_block_sparse_attn_raster_fused(const void* q, const void* k, const void* v, const usv_shape* shape,
                                              const usv_raster* view, const int32_t* idx, const int32_t* cnt,
                                              int32_t kmax, float scale, const float* coarse, const void* gate_fine,
                                              const void* gate_coarse, int32_t out_dtype, void* out, float* lse,
                                              void* stream) {
  usv::Dims s;
  usv::RasterArgs ras;
  USV_TRY(check_shape(shape, true, &s));
  if (!s.bf16) return fail(USV_ERR_UNSUPPORTED, "the raster-order attention takes bf16 inputs");
  if (out_dtype != USV_BF16 && out_dtype != USV_F32) return fail(USV_ERR_UNSUPPORTED, "out_dtype must be USV_BF16 or USV_F32");
  USV_TRY(check_raster(view, s, out_dtype == USV_F32 ? 4 : 2, &ras));
  USV_TRY(check_ptr(q, "q"));
  USV_TRY(check_ptr(k, "k"));
  USV_TRY(check_ptr(v, "v"));
  USV_TRY(check_ptr(idx, "idx"));
  USV_TRY(check_ptr(cnt, "cnt"));
  USV_TRY(check_ptr(out, "out"));
  if (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) return fail(USV_ERR_INVALID_ARG, "lse is not 4-byte aligned");
  if (kmax < 1 || kmax > s.nb) return fail(USV_ERR_INVALID_ARG, "kmax (%d) must be in [1, blocks = %d]", kmax, s.nb);
  if (std::isnan(scale) || std::isinf(scale)) return fail(USV_ERR_INVALID_ARG, "scale must be finite");
  if (!coarse && (gate_fine || gate_coarse)) return fail(USV_ERR_INVALID_ARG, "gates without coarse");
  if (coarse && !aligned16(coarse)) return fail(USV_ERR_INVALID_ARG, "coarse is not 16-byte aligned");
  if (gate_fine && !aligned16(gate_fine)) return fail(USV_ERR_INVALID_ARG, "gate_fine is not 16-byte aligned");
  if (gate_coarse && !aligned16(gate_coarse)) return fail(USV_ERR_INVALID_ARG, "gate_coarse is not 16-byte aligned");
  if (scale <= 0.f) scale = 1.0f / std::sqrt((float)s.d);
  const usv::FuseArgs fuse{coarse, static_cast<const uint16_t*>(gate_fine), static_cast<const uint16_t*>(gate_coarse)};
  if (view->work_order) USV_TRY(check_ptr(view->work_order, "work_order"));
  return hip_result(usv::launch_attn_bf16_raster(q, k, v, s, ras, idx, cnt, kmax, scale, out, out_dtype == USV_F32, lse,
                                                 fuse, static_cast<hipStream_t>(stream), view->work_order),
                    "usv_block_sparse_attn_raster launch");
}

usv_status usv_cube_token_order(const usv_grid* grid, int32_t* order) {
  usv::CubeGrid g;
  USV_TRY(check_grid(grid, nullptr, &g));
  if (!order) return fail(USV_ERR_INVALID_ARG, "order is NULL");
  for (int t = 0; t < g.T; ++t)
    for (int h = 0; h < g.H; ++h)
      for (int w = 0; w < g.W; ++w) order[usv::cube_position(g, t, h, w)] = (t * g.H + h) * g.W + w;
  g_err[0] = '\0';
  return USV_OK;
}

usv_status usv_cube_gather(const void* raster, const usv_strides* strides, const usv_shape* shape,
                           const usv_grid* grid, void* cube, void* stream) {
  usv::Dims s;
  usv::CubeGrid g;
  long long sb[3];
  USV_TRY(check_shape(shape, true, &s));
  USV_TRY(check_grid(grid, shape, &g));
  USV_TRY(check_strides(strides, s, sb));
  USV_TRY(check_ptr(raster, "raster"));
  USV_TRY(check_ptr(cube, "cube"));
  return hip_result(usv::launch_cube_move(true, raster, cube, g, s, sb[0], sb[1], sb[2], static_cast<hipStream_t>(stream)),
                    "usv_cube_gather launch");
}

usv_status usv_cube_scatter(const void* cube, const usv_shape* shape, const usv_grid* grid, void* raster,
                            const usv_strides* strides, void* stream) {
  usv::Dims s;
  usv::CubeGrid g;
  long long sb[3];
  USV_TRY(check_shape(shape, true, &s));
  USV_TRY(check_grid(grid, shape, &g));
  USV_TRY(check_strides(strides, s, sb));
  USV_TRY(check_ptr(cube, "cube"));
  USV_TRY(check_ptr(raster, "raster"));
  return hip_result(usv::launch_cube_move(false, cube, raster, g, s, sb[0], sb[1], sb[2], static_cast<hipStream_t>(stream)),
                    "usv_cube_scatter launch");
}

const char* usv_status_string(int32_t status) {
  switch (status) {
    case USV_OK: return "USV_OK";
    case USV_ERR_INVALID_ARG: return "USV_ERR_INVALID_ARG";
    case USV_ERR_UNSUPPORTED: return "USV_ERR_UNSUPPORTED";
    case USV_ERR_WORKSPACE: return "USV_ERR_WORKSPACE";
    case USV_ERR_HIP: return "USV_ERR_HIP";
    default: return "USV_ERR_UNKNOWN";
  }
}

const char* usv_last_error(void) { return g_err; }

}  // extern "C"
