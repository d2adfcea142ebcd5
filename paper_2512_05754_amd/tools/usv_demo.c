/*
 * The three stages from plain C: no Python, no torch, only the C ABI of libusv.so and the HIP
 * runtime for device memory.  Built by `python -m paper_2512_05754_amd.build` with gcc -std=c99.
 *
 *   usv_demo DIR
 *
 * reads   DIR/shape.txt   "B Hh N Nv d keep"  (bf16 inputs; N a multiple of 64)
 *         DIR/q.bin, k.bin, v.bin             [B, Hh, N, d] bf16 bit patterns, cube-major token order
 * writes  DIR/scores.bin  [B, Hh, nb, nb] fp32        (usv_block_scores)
 *         DIR/idx.bin     [B, Hh, nb, keep] int32     (usv_select_topk)
 *         DIR/cnt.bin     [B, Hh, nb] int32
 *         DIR/out.bin     [B, Hh, N, d] fp32          (usv_block_sparse_attn, fp32 output)
 * and prints one line per stage.  Exit status 0 on success, 1 on any error (message on stderr).
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "usv.h"

static int fail(const char* what, const char* detail) {
  fprintf(stderr, "usv_demo: %s: %s\n", what, detail);
  return 1;
}

#define HIP_TRY(call)                                                  \
  do {                                                                 \
    hipError_t e_ = (call);                                            \
    if (e_ != hipSuccess) return fail(#call, hipGetErrorString(e_));   \
  } while (0)

#define USV_TRY(call)                                                  \
  do {                                                                 \
    usv_status s_ = (call);                                            \
    if (s_ != USV_OK) return fail(#call, usv_last_error());            \
  } while (0)

static void* read_file(const char* dir, const char* name, size_t bytes) {
  char path[4096];
  snprintf(path, sizeof path, "%s/%s", dir, name);
  FILE* f = fopen(path, "rb");
  if (!f) return NULL;
  void* buf = malloc(bytes);
  if (buf && fread(buf, 1, bytes, f) != bytes) {
    free(buf);
    buf = NULL;
  }
  fclose(f);
  return buf;
}

static int write_file(const char* dir, const char* name, const void* buf, size_t bytes) {
  char path[4096];
  snprintf(path, sizeof path, "%s/%s", dir, name);
  FILE* f = fopen(path, "wb");
  if (!f) return 1;
  const int bad = fwrite(buf, 1, bytes, f) != bytes;
  return fclose(f) != 0 || bad;
}

/* device buffer -> file */
static int dump(const char* dir, const char* name, const void* dev, size_t bytes) {
  void* host = malloc(bytes);
  if (!host) return fail(name, "out of host memory");
  HIP_TRY(hipMemcpy(host, dev, bytes, hipMemcpyDeviceToHost));
  const int bad = write_file(dir, name, host, bytes);
  free(host);
  return bad ? fail(name, "cannot write") : 0;
}

int main(int argc, char** argv) {
  if (argc != 2) return fail("usage", "usv_demo DIR");
  const char* dir = argv[1];
  char path[4096];
  snprintf(path, sizeof path, "%s/shape.txt", dir);
  FILE* f = fopen(path, "r");
  int B, Hh, N, Nv, d, keep;
  if (!f || fscanf(f, "%d %d %d %d %d %d", &B, &Hh, &N, &Nv, &d, &keep) != 6) return fail(path, "cannot read six integers");
  fclose(f);

  usv_shape shape;
  memset(&shape, 0, sizeof shape);
  shape.batch = B;
  shape.heads = Hh;
  shape.seq_len = N;
  shape.seq_valid = Nv;
  shape.head_dim = d;
  shape.block = 64;
  shape.dtype = USV_BF16;
  const size_t ws_bytes = usv_workspace_bytes(&shape);
  if (ws_bytes == 0) return fail("usv_workspace_bytes", "the library rejects this shape");
  const size_t nb = (size_t)N / 64, bh = (size_t)B * Hh;
  const size_t in_bytes = bh * N * d * 2, s_bytes = bh * nb * nb * 4, idx_bytes = bh * nb * keep * 4, cnt_bytes = bh * nb * 4,
               out_bytes = bh * N * d * 4;

  void *q, *k, *v, *ws, *scores, *idx, *cnt, *out;
  HIP_TRY(hipMalloc(&q, in_bytes));
  HIP_TRY(hipMalloc(&k, in_bytes));
  HIP_TRY(hipMalloc(&v, in_bytes));
  HIP_TRY(hipMalloc(&ws, ws_bytes));
  HIP_TRY(hipMalloc(&scores, s_bytes));
  HIP_TRY(hipMalloc(&idx, idx_bytes));
  HIP_TRY(hipMalloc(&cnt, cnt_bytes));
  HIP_TRY(hipMalloc(&out, out_bytes));
  const char* names[3] = {"q.bin", "k.bin", "v.bin"};
  void* dev[3];
  dev[0] = q;
  dev[1] = k;
  dev[2] = v;
  for (int t = 0; t < 3; ++t) {
    void* host = read_file(dir, names[t], in_bytes);
    if (!host) return fail(names[t], "cannot read");
    HIP_TRY(hipMemcpy(dev[t], host, in_bytes, hipMemcpyHostToDevice));
    free(host);
  }

  hipStream_t stream;
  HIP_TRY(hipStreamCreate(&stream));
  USV_TRY(usv_block_scores(q, k, &shape, (float*)scores, ws, ws_bytes, stream));
  USV_TRY(usv_select_topk((const float*)scores, &shape, keep, NULL, keep, (int32_t*)idx, (int32_t*)cnt, stream));
  USV_TRY(usv_block_sparse_attn(q, k, v, &shape, (const int32_t*)idx, (const int32_t*)cnt, keep, 0.0f, USV_F32, out, NULL, stream));
  HIP_TRY(hipStreamSynchronize(stream));
  printf("usv_block_scores      -> scores.bin  [%d, %d, %zu, %zu] fp32\n", B, Hh, nb, nb);
  printf("usv_select_topk       -> idx.bin     [%d, %d, %zu, %d] int32, cnt.bin\n", B, Hh, nb, keep);
  printf("usv_block_sparse_attn -> out.bin     [%d, %d, %d, %d] fp32\n", B, Hh, N, d);

  if (dump(dir, "scores.bin", scores, s_bytes) || dump(dir, "idx.bin", idx, idx_bytes) || dump(dir, "cnt.bin", cnt, cnt_bytes) ||
      dump(dir, "out.bin", out, out_bytes))
    return 1;
  HIP_TRY(hipStreamDestroy(stream));
  void* all[8];
  all[0] = q; all[1] = k; all[2] = v; all[3] = ws; all[4] = scores; all[5] = idx; all[6] = cnt; all[7] = out;
  for (int t = 0; t < 8; ++t) HIP_TRY(hipFree(all[t]));
  return 0;
}
