// Stand-alone probe: what the bf16 matrix pipe of this GPU sustains with nothing else going on.
//
// 512 workgroups x 8 wavefronts run v_mfma_f32_32x32x16_bf16 back to back on four independent
// accumulators, operands held in registers (no LDS, no memory traffic in the loop). The operand
// bits are taken from memory once: all 1.0, all zeros, or random bf16 values. The published peak
// (2.5 PFLOP/s dense bf16) is reached with constant operands; with random operands the chip lowers
// its clock (power management), which bounds any real kernel: attention roofline fractions in this
// repository are quoted against the published peak, and this probe says how much of it is reachable.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(512) void mfma_loop(const u32x4* src, float* out, int iters) {
  bf16x8 a[8], b[8];
  for (int i = 0; i < 8; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, src[(threadIdx.x * 16 + i) & 8191]);
    b[i] = __builtin_bit_cast(bf16x8, src[(threadIdx.x * 16 + 8 + i) & 8191]);
  }
  f32x16 acc[4];
  for (int n = 0; n < 4; ++n)
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + n) & 7], b[i], acc[n], 0, 0, 0);
  }
  float s = 0;
  for (int n = 0; n < 4; ++n)
    for (int r = 0; r < 16; ++r) s += acc[n][r];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

#define CHECK(x)                                                              \
  do {                                                                        \
    hipError_t e_ = (x);                                                      \
    if (e_ != hipSuccess) {                                                   \
      fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                 \
      return 1;                                                               \
    }                                                                         \
  } while (0)

int main() {
  u32x4* src;
  float* out;
  CHECK(hipMalloc(&src, 8192 * 16));
  CHECK(hipMalloc(&out, 512 * 512 * 4));
  unsigned* h = (unsigned*)malloc(8192 * 16);
  const char* names[3] = {"all 1.0", "all zeros", "random bf16 (sign, 7-bit mantissa, exponent 120..127)"};
  srand(1);
  for (int mode = 0; mode < 3; ++mode) {
    for (int i = 0; i < 8192 * 4; ++i) {
      if (mode == 0) h[i] = 0x3f803f80u;
      else if (mode == 1) h[i] = 0;
      else {
        const unsigned lo = (rand() & 0x807f) | ((120 + rand() % 8) << 7);
        const unsigned hi = (rand() & 0x807f) | ((120 + rand() % 8) << 7);
        h[i] = (hi << 16) | (lo & 0xffff);
      }
    }
    CHECK(hipMemcpy(src, h, 8192 * 16, hipMemcpyHostToDevice));
    const int iters = 4000;  // 32 MFMAs per iteration and wavefront
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    hipLaunchKernelGGL(mfma_loop, dim3(512), dim3(512), 0, 0, src, out, iters);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    for (int r = 0; r < 5; ++r) hipLaunchKernelGGL(mfma_loop, dim3(512), dim3(512), 0, 0, src, out, iters);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    ms /= 5;
    const double flops = 512.0 * 8 * iters * 32 * 32768.0;
    printf("operands %s: %.3f ms per launch, %.1f TFLOP/s (%.1f %% of 2500)\n", names[mode], ms, flops / ms / 1e9,
           flops / ms / 1e9 / 25.0);
  }
  return 0;
}
