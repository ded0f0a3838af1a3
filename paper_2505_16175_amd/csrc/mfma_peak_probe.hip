// Stand-alone probe: what the bf16 matrix pipe of this GPU sustains with nothing else going on.
//
// 512 workgroups x 8 wavefronts run v_mfma_f32_32x32x16_bf16 back to back on four independent
// accumulators, operands held in registers (no LDS, no memory traffic in the loop). The operand
// bits are taken from memory once: all 1.0, all zeros, or random bf16 values. The published peak
// (2.5 PFLOP/s dense bf16) is reached with constant operands; with random operands the chip lowers
// its clock (power management), which bounds any real kernel: attention roofline fractions in this
// repository are quoted against the published peak, and this probe says how much of it is reachable.
// A second part (overlap_loop below) measures how far vector work hides under another wavefront's MFMAs.
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

// Second question: does the vector work of one wavefront run under the MFMAs of another wavefront of the same
// SIMD? 16 workgroups of 8 wavefronts (16 CUs, far below any power limit; wavefronts w and w+4 share a SIMD).
// mode bits: 1 = wavefronts 0..3 run 32 MFMAs per iteration, 4 = wavefronts 4..7 do, 2 = wavefronts 4..7 run a
// block of ~130 vector operations with 32 exp2 (the size of one tile's softmax), 8 = wavefronts 0..3 do.
__global__ __launch_bounds__(512) void overlap_loop(float* out, int iters, int mode, float seed) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const bool lo = wave < 4;
  const bool do_mfma = lo ? (mode & 1) : (mode & 4);
  const bool do_valu = lo ? (mode & 8) : (mode & 2);
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(seed * (lane + i));
    b[i] = (__bf16)(seed * (lane * 3 + i));
  }
  f32x16 acc[4];
  for (int n = 0; n < 4; ++n)
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  float v[16];
  for (int i = 0; i < 16; ++i) v[i] = seed * (lane + i);
  // mode bit 16: wavefronts 4..7 run their vector block BEFORE their MFMAs (opposite phase order to wavefronts 0..3);
  // mode bit 32: a workgroup barrier per iteration (what a shared tile ring imposes)
  const bool valu_first = (mode & 16) && !lo;
  const bool barrier = mode & 32;
  const int barrier_every = (mode & 64) ? 2 : ((mode & 128) ? 4 : 1);  // with bit 32: a barrier every that many iterations
  for (int it = 0; it < iters; ++it) {
    if (do_valu && valu_first) {
#pragma unroll
      for (int rep = 0; rep < 2; ++rep)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float x = fmaf(v[i], 0.999f, -0.25f);
          x = __builtin_amdgcn_exp2f(x);
          v[i] = fmaxf(x, v[(i + 1) & 15]) * 0.5f + 0.125f;
        }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (do_mfma) {
#pragma unroll
      for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (do_valu && !valu_first) {
#pragma unroll
      for (int rep = 0; rep < 2; ++rep)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float x = fmaf(v[i], 0.999f, -0.25f);
          x = __builtin_amdgcn_exp2f(x);
          v[i] = fmaxf(x, v[(i + 1) & 15]) * 0.5f + 0.125f;
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (barrier && (it + 1) % barrier_every == 0) __syncthreads();
  }
  float s = 0.f;
  for (int n = 0; n < 4; ++n)
    for (int r = 0; r < 16; ++r) s += acc[n][r];
  for (int i = 0; i < 16; ++i) s += v[i];
  out[blockIdx.x * 512 + threadIdx.x] = s;
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
  // co-execution of MFMA and vector work on one SIMD
  const int modes[] = {1, 2, 3, 5, 10, 9, 15, 15 | 32, 15 | 32 | 64, 15 | 32 | 128, 15 | 16, 15 | 16 | 32, 15 | 16 | 32 | 64};
  const char* what[] = {"wavefronts 0-3: MFMAs, 4-7 idle", "wavefronts 4-7: vector block, 0-3 idle",
                        "wavefronts 0-3: MFMAs, 4-7: vector block", "all 8: MFMAs", "all 8: vector block",
                        "wavefronts 0-3: MFMAs then vector block, 4-7 idle", "all 8: MFMAs then vector block",
                        "all 8: MFMAs then vector block, barrier per iteration",
                        "all 8: MFMAs then vector block, barrier every 2nd",
                        "all 8: MFMAs then vector block, barrier every 4th",
                        "0-3: MFMAs then vector, 4-7: vector then MFMAs",
                        "0-3: MFMAs then vector, 4-7: vector then MFMAs, barrier",
                        "0-3: MFMAs then vector, 4-7: vector then MFMAs, barrier every 2nd"};
  const int it2 = 20000;
  for (int m = 0; m < 13; ++m) {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    hipLaunchKernelGGL(overlap_loop, dim3(16), dim3(512), 0, 0, out, 100, modes[m], 0.001f);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL(overlap_loop, dim3(16), dim3(512), 0, 0, out, it2, modes[m], 0.001f);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("16 CUs, %-52s: %.1f ns per iteration (32 MFMAs and/or ~130 vector ops per wavefront)\n", what[m],
           ms * 1e6 / it2);
  }
  return 0;
}
