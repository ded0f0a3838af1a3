// Small HBM-bound kernels of the decoder layer around the path: RMSNorm and the table of rotary angles.
#include "qp_internal.h"

namespace qp {

// y[t][i] = x[t][i] / sqrt(mean_i x[t][i]^2 + eps) * w[i], f32 arithmetic, one rounding to bf16 at the store.
// One wavefront per token. Rows of up to RN_REG * 512 elements (8192 for RN_REG = 16) stay in registers between the
// sum of squares and the scaling, so the row is read once; longer rows are read a second time (from cache).
constexpr int RN_WAVES = 4;
constexpr int RN_REG = 16;  // 16-byte chunks per lane held in registers
__global__ __launch_bounds__(RN_WAVES * 64) void rms_norm_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w,
                                                                 bf16_t* __restrict__ out, int n_tokens, int d_model,
                                                                 float eps) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * RN_WAVES + (threadIdx.x >> 6);
  if (t >= n_tokens) return;
  const int chunks = d_model / 8;
  const uint4* xr = (const uint4*)(x + (size_t)t * d_model);
  const uint4* wr = (const uint4*)w;
  uint4* orow = (uint4*)(out + (size_t)t * d_model);
  const bool in_regs = chunks <= RN_REG * 64;
  uint4 held[RN_REG];
  float ss = 0.f;
  if (in_regs) {
#pragma unroll
    for (int i = 0; i < RN_REG; ++i) {
      const int c = lane + 64 * i;
      held[i] = c < chunks ? xr[c] : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int i = 0; i < RN_REG; ++i) {
      float f[8];
      widen16<bf16_t>(held[i], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss = fmaf(f[e], f[e], ss);
    }
  } else {
    for (int c = lane; c < chunks; c += 64) {
      float f[8];
      widen16<bf16_t>(xr[c], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss = fmaf(f[e], f[e], ss);
    }
  }
  ss = wave_sum(ss);
  const float inv = 1.f / sqrtf(ss / (float)d_model + eps);
  auto scale_store = [&](int c, const uint4& raw) {
    float f[8], g[8];
    widen16<bf16_t>(raw, f);
    widen16<bf16_t>(wr[c], g);
    uint32_t p[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      p[e] = (uint32_t)f32_to_bf16_rne(f[2 * e] * inv * g[2 * e]) | ((uint32_t)f32_to_bf16_rne(f[2 * e + 1] * inv * g[2 * e + 1]) << 16);
    orow[c] = make_uint4(p[0], p[1], p[2], p[3]);
  };
  if (in_regs) {
#pragma unroll
    for (int i = 0; i < RN_REG; ++i) {
      const int c = lane + 64 * i;
      if (c < chunks) scale_store(c, held[i]);
    }
  } else {
    for (int c = lane; c < chunks; c += 64) scale_store(c, xr[c]);
  }
}

void launch_rms_norm(const void* x, const void* w, void* out, int n_tokens, int d_model, float eps, hipStream_t s) {
  hipLaunchKernelGGL(rms_norm_kernel, dim3((n_tokens + RN_WAVES - 1) / RN_WAVES), dim3(RN_WAVES * 64), 0, s,
                     (const bf16_t*)x, (const bf16_t*)w, (bf16_t*)out, n_tokens, d_model, eps);
}

// cos_sin[t][i] = (cos, sin)(pos[axis(i)][t] * theta^(-i/64)) for the 64 rotation frequencies of head_dim 128;
// frequencies [0, s0) use position axis 0, [s0, s0+s1) axis 1, the rest axis 2. The angle (up to ~1e5 rad for long
// videos) and its sine/cosine are evaluated in f64 and rounded once, so the table is as exact as f32 holds.
__global__ __launch_bounds__(256) void rope_table_kernel(const int32_t* __restrict__ pos, long axis_stride, int n_tokens,
                                                         float theta, int s0, int s1, float2* __restrict__ cos_sin) {
  const int id = blockIdx.x * 256 + threadIdx.x;
  if (id >= n_tokens * 64) return;
  const int t = id >> 6, i = id & 63;
  const int axis = i < s0 ? 0 : (i < s0 + s1 ? 1 : 2);
  const double ang = (double)pos[axis * axis_stride + t] * exp2(-(double)i / 64.0 * log2((double)theta));
  double sn, cs;
  sincos(ang, &sn, &cs);
  cos_sin[id] = make_float2((float)cs, (float)sn);
}

void launch_rope_table(const int32_t* pos, long axis_stride, int n_tokens, float theta, int s0, int s1, float* cos_sin,
                       hipStream_t s) {
  hipLaunchKernelGGL(rope_table_kernel, dim3((n_tokens * 64 + 255) / 256), dim3(256), 0, s, pos, axis_stride, n_tokens,
                     theta, s0, s1, (float2*)cos_sin);
}

}  // namespace qp
