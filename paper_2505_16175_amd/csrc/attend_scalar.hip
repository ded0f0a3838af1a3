// Scalar (non-MFMA) group attention: f32 and bf16 inputs, f32 arithmetic.
//
// One wavefront owns one query row (token i of query head qh). Its 64 lanes take the
// visible keys round-robin (lane l: keys l, l+64, ...), each lane running its own online
// softmax (running max m, denominator l, d accumulators); the 64 partial states are
// merged once at the end. The visible keys of a row are the C cache entries of its KV head
// followed by group tokens 0..i (Sec. 3.2: pruned cache + own group, causal).
//
// This kernel is the f32 path (tiny config) and the fallback for layouts the MFMA kernel
// does not take; it is not tuned.
#include "qp_internal.h"

namespace qp {

template <typename T, int D>
__global__ __launch_bounds__(256) void attend_scalar_kernel(AttendArgs a) {
  constexpr int WAVES = 4;
  constexpr int PER = Elem<T>::kPer16B;   // elements per 16-byte chunk
  constexpr int CHUNKS = D / PER;
  __shared__ float q_lds[WAVES][D];

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * WAVES + wave;  // group token (query row)
  const int qh = blockIdx.y;
  const int r = a.h_q / a.h_kv;
  const int h = qh / r;
  const bool active = i < a.n_g;            // whole wave agrees

  if (active) {
    const T* qrow = (const T*)a.q + ((size_t)i * a.h_q + qh) * D;
    for (int c = lane; c < CHUNKS; c += 64) {
      uint4 raw = *(const uint4*)(qrow + c * PER);
      float tmp[PER];
      widen16<T>(raw, tmp);
#pragma unroll
      for (int e = 0; e < PER; ++e) q_lds[wave][c * PER + e] = tmp[e];
    }
  }
  __syncthreads();
  if (!active) return;

  float m = -INFINITY, l = 0.f;
  float acc[D];
#pragma unroll
  for (int c = 0; c < D; ++c) acc[c] = 0.f;

  const int n_keys = a.c + i + 1;
  const T* ck = (const T*)a.ck + (size_t)h * a.cap * D;
  const T* cv = (const T*)a.cv + (size_t)h * a.cap * D;
  const T* gk = (const T*)a.k + (size_t)h * D;
  const T* gv = (const T*)a.v + (size_t)h * D;
  const size_t gstride = (size_t)a.h_kv * D;

  for (int j = lane; j < n_keys; j += 64) {
    const T* krow;
    const T* vrow;
    if (j < a.c) {
      krow = ck + (size_t)j * D;
      vrow = cv + (size_t)j * D;
    } else {
      krow = gk + (size_t)(j - a.c) * gstride;
      vrow = gv + (size_t)(j - a.c) * gstride;
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      uint4 raw = *(const uint4*)(krow + c * PER);
      float kv[PER];
      widen16<T>(raw, kv);
#pragma unroll
      for (int e = 0; e < PER; ++e) s = fmaf(q_lds[wave][c * PER + e], kv[e], s);
    }
    s *= a.scale_log2;
    if (s > m) {
      const float alpha = exp2f(m - s);    // exp2(-inf) = 0 on the first key
      l *= alpha;
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] *= alpha;
      m = s;
    }
    const float p = exp2f(s - m);
    l += p;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      uint4 raw = *(const uint4*)(vrow + c * PER);
      float vv[PER];
      widen16<T>(raw, vv);
#pragma unroll
      for (int e = 0; e < PER; ++e) acc[c * PER + e] = fmaf(p, vv[e], acc[c * PER + e]);
    }
  }

  // merge the 64 lane states
  const float mw = wave_max(m);             // finite: every row sees at least itself
  const float f = exp2f(m - mw);            // lanes without keys: exp2(-inf) = 0
  const float lw = wave_sum(l * f);
  const float inv = 1.f / lw;
  constexpr int OUT_PER_LANE = (D + 63) / 64;
  float o[OUT_PER_LANE];
#pragma unroll
  for (int c = 0; c < D; ++c) {
    const float t = wave_sum(acc[c] * f);
    if (lane == (c & 63)) o[c >> 6] = t * inv;
  }
  T* orow = (T*)a.out + ((size_t)i * a.h_q + qh) * D;
#pragma unroll
  for (int e = 0; e < OUT_PER_LANE; ++e) {
    const int c = e * 64 + lane;
    if (c < D) store_elem<T>(orow + c, o[e]);
  }
  if (a.lse != nullptr && lane == 0) a.lse[(size_t)qh * a.n_g + i] = (mw + log2f(lw)) * 0.6931471805599453f;
}

void launch_attend_scalar(const AttendArgs& a, int dtype, hipStream_t s) {
  dim3 grid((a.n_g + 3) / 4, a.h_q), block(256);
  if (dtype == QP_F32) {
    if (a.d == 64) hipLaunchKernelGGL((attend_scalar_kernel<float, 64>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((attend_scalar_kernel<float, 128>), grid, block, 0, s, a);
  } else {
    if (a.d == 64) hipLaunchKernelGGL((attend_scalar_kernel<bf16_t, 64>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((attend_scalar_kernel<bf16_t, 128>), grid, block, 0, s, a);
  }
}

}  // namespace qp
