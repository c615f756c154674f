// Stand-alone probe: what the matrix cores of this GPU sustain on
// v_mfma_f32_32x32x16_bf16 alone - no memory traffic, no LDS, no vector ALU
// work inside the loop - with all-zero operands and with random N(0,1) bf16
// operands.  The clock the power management grants depends on the operand
// data, so the second figure, not the data-sheet peak, is the ceiling a kernel
// working on real activations can approach.
//
// Usage: mfma_peak_probe [launches per measurement]   (one JSON object on stdout)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int WORDS = 1 << 20;     // 16-byte operand words in the data buffer
constexpr int GRID = 512;          // 256 CUs x 2 workgroups
constexpr int THREADS = 256;       // 4 wavefronts: two per SIMD with two workgroups per CU
constexpr int MFMA_PER_ITER = 8;

__global__ __launch_bounds__(THREADS, 2) void mfma_loop(const u32x4 *data, float *out, int iters, int *clk) {
  const int tid = threadIdx.x + blockIdx.x * blockDim.x;
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, data[(tid * 16 + i) & (WORDS - 1)]);
    b[i] = __builtin_bit_cast(bf16x8, data[(tid * 16 + 8 + i) & (WORDS - 1)]);
  }
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
  const unsigned long long c0 = __builtin_amdgcn_s_memtime(), t0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < MFMA_PER_ITER; ++j)
      acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + 3) & 7], acc[j & 3], 0, 0, 0);
  }
  const unsigned long long c1 = __builtin_amdgcn_s_memtime(), t1 = __builtin_amdgcn_s_memrealtime();
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[j][v];
  out[tid] = s;
  if (tid == 0) {  // shader-clock cycles and 100 MHz ticks of the loop
    clk[0] = (int)(c1 - c0);
    clk[1] = (int)(t1 - t0);
  }
}

#define CHECK(x)                                                                    \
  do {                                                                              \
    hipError_t e_ = (x);                                                            \
    if (e_ != hipSuccess) {                                                         \
      fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                       \
      return 1;                                                                     \
    }                                                                               \
  } while (0)

int main(int argc, char **argv) {
  const int launches = argc > 1 ? atoi(argv[1]) : 60;
  if (launches <= 0) return 2;
  std::vector<uint32_t> h((size_t)WORDS * 4);
  u32x4 *d;
  float *out;
  int *clk;
  CHECK(hipMalloc(&d, (size_t)WORDS * 16));
  CHECK(hipMalloc(&out, (size_t)GRID * THREADS * 4));
  CHECK(hipMalloc(&clk, 8));
  std::mt19937 rng(1);
  std::normal_distribution<float> nd(0.f, 1.f);
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  const int iters = 40000;
  printf("{");
  for (int mode = 0; mode < 2; ++mode) {
    for (auto &w : h) {
      if (mode == 0) {
        w = 0;
      } else {  // two bf16 (truncated fp32) per word
        const float x = nd(rng), y = nd(rng);
        uint32_t bx, by;
        memcpy(&bx, &x, 4);
        memcpy(&by, &y, 4);
        w = (bx >> 16) | (by & 0xffff0000u);
      }
    }
    CHECK(hipMemcpy(d, h.data(), (size_t)WORDS * 16, hipMemcpyHostToDevice));
    float ms = 0.f;
    for (int rep = 0; rep < 2; ++rep) {  // the second measurement is reported: clocks have settled
      CHECK(hipEventRecord(e0));
      for (int l = 0; l < launches; ++l) hipLaunchKernelGGL(mfma_loop, dim3(GRID), dim3(THREADS), 0, 0, d, out, iters, clk);
      CHECK(hipGetLastError());
      CHECK(hipEventRecord(e1));
      CHECK(hipEventSynchronize(e1));
      CHECK(hipEventElapsedTime(&ms, e0, e1));
    }
    int hc[2];
    CHECK(hipMemcpy(hc, clk, 8, hipMemcpyDeviceToHost));
    const double flops = (double)launches * GRID * (THREADS / 64) * (double)iters * MFMA_PER_ITER * 32768.0;
    printf("%s\"%s\": {\"tflops\": %.1f, \"sclk_mhz\": %.0f}", mode ? ", " : "", mode ? "random" : "zeros",
           flops / ms / 1e9, 100.0 * hc[0] / hc[1]);
  }
  printf("}\n");
  return 0;
}
