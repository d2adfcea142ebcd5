// Measures what an MFMA-only loop sustains on this GPU with either bf16 shape (v_mfma_f32_32x32x16_bf16:
// four independent accumulators per wave; v_mfma_f32_16x16x32_bf16, the one the attention kernel uses:
// sixteen), 2 or 3 waves per SIMD, no memory traffic.  The rate depends on the operand
// DATA: with constant operands the clock stays near its maximum, with operands distributed like real
// activations the chip throttles (power), so both are reported.  This is the practical ceiling the
// attention kernel's roofline fraction should be read against; the nominal peak is 2.5 PFLOP/s.
// Usage: mfma_peak    prints one JSON object.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

// SHAPE 0: 32x32x16, 16 MFMAs per trip.  SHAPE 1: 16x16x32, 64 MFMAs per trip (twice the flops per trip).
template <int SHAPE>
__global__ __launch_bounds__(256) void mfma_loop(const bf16x8* data, float* out, int iters) {
  bf16x8 a[4], b[4];
  for (int i = 0; i < 4; i++) {
    a[i] = data[(threadIdx.x * 8 + i) % 4096];
    b[i] = data[(threadIdx.x * 8 + 4 + i) % 4096];
  }
  float s = 0.f;
  if constexpr (SHAPE == 0) {
    f32x16 acc[4];
    for (int j = 0; j < 4; j++)
      for (int r = 0; r < 16; r++) acc[j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int u = 0; u < 4; u++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + u) & 3], acc[j], 0, 0, 0);
    }
    for (int j = 0; j < 4; j++)
      for (int r = 0; r < 16; r++) s += acc[j][r];
  } else {
    f32x4 acc[16];
    for (int j = 0; j < 16; j++)
      for (int r = 0; r < 4; r++) acc[j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int u = 0; u < 4; u++)
#pragma unroll
        for (int j = 0; j < 16; j++)
          acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j & 3], b[((j >> 2) + u) & 3], acc[j], 0, 0, 0);
    }
    for (int j = 0; j < 16; j++)
      for (int r = 0; r < 4; r++) s += acc[j][r];
  }
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

static unsigned short to_bf16(float f) {
  unsigned u;
  memcpy(&u, &f, 4);
  return (unsigned short)((u + 0x7fff + ((u >> 16) & 1)) >> 16);
}

static float gauss() {  // Irwin-Hall approximation of N(0,1): enough for a power test
  float s = 0.f;
  for (int i = 0; i < 12; i++) s += (float)rand() / (float)RAND_MAX;
  return s - 6.f;
}

#define CK(x)                                                         \
  do {                                                                \
    hipError_t e_ = (x);                                              \
    if (e_ != hipSuccess) {                                           \
      fprintf(stderr, "HIP error: %s\n", hipGetErrorString(e_));      \
      return 1;                                                       \
    }                                                                 \
  } while (0)

int main(int argc, char** argv) {
  (void)argc;
  (void)argv;
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  const int cus = prop.multiProcessorCount;
  float* out;
  bf16x8* data;
  CK(hipMalloc(&out, (size_t)cus * 3 * 256 * sizeof(float)));
  CK(hipMalloc(&data, 4096 * sizeof(bf16x8)));
  unsigned short* host = (unsigned short*)malloc(4096 * 16);
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  srand(1);
  double best[2][2] = {{0, 0}, {0, 0}};  // [shape][operands]
  for (int shape = 0; shape < 2; ++shape)
  for (int mode = 0; mode < 2; ++mode) {
    for (int i = 0; i < 4096 * 8; i++) host[i] = to_bf16(mode == 0 ? 1.0f : gauss() * 2.2f);
    CK(hipMemcpy(data, host, 4096 * 16, hipMemcpyHostToDevice));
    for (int waves = 2; waves <= 3; ++waves) {
      const int grid = cus * waves, iters = 5000;
      auto launch = [&](int n) {
        if (shape == 0)
          mfma_loop<0><<<grid, 256>>>(data, out, n);
        else
          mfma_loop<1><<<grid, 256>>>(data, out, n);
      };
      launch(1000);  // warm the clocks
      CK(hipDeviceSynchronize());
      CK(hipEventRecord(e0));
      launch(iters);
      CK(hipEventRecord(e1));
      CK(hipEventSynchronize(e1));
      float ms;
      CK(hipEventElapsedTime(&ms, e0, e1));
      const double flop_per_trip = shape == 0 ? 16 * 2.0 * 32 * 32 * 16 : 64 * 2.0 * 16 * 16 * 32;
      const double tflops = (double)grid * 4 /*waves*/ * iters * flop_per_trip / ms / 1e9;
      if (tflops > best[shape][mode]) best[shape][mode] = tflops;
    }
  }
  // the headline pair is the shape the attention kernel issues
  printf("{\"instruction\": \"v_mfma_f32_16x16x32_bf16\", \"compute_units\": %d, "
         "\"constant_operands_tflops\": %.1f, \"gaussian_operands_tflops\": %.1f, "
         "\"v_mfma_f32_32x32x16_bf16\": {\"constant_operands_tflops\": %.1f, \"gaussian_operands_tflops\": %.1f}}\n",
         cus, best[1][0], best[1][1], best[0][0], best[0][1]);
  return 0;
}
