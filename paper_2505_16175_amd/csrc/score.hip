// Importance scores of a group's new KV entries (the functions listed under Eq. 2, Sec. 3.2).
//
//   Key Norms (small):  s[h][j] = -||K_g[j,h,:]||_2
//   Value Norms:        s[h][j] = +||V_g[j,h,:]||_2
//   Attention Scores:   s[h][j] = sum over query heads qh of KV head h and window rows t of
//                       softmax_j(scale * Q_win[t,qh,:] . K_g[j,h,:])   (softmax over the group's keys)
//
// Norms: a row of d elements is 256 bytes (bf16 d=128, f32 d=64) or a multiple of 16 bytes in
// general; LPR = row bytes / 16 lanes load one 16-byte chunk each, square-accumulate in f32 and
// finish with an xor-shuffle reduction inside the LPR-lane group; every lane keeps four rows' loads in
// flight. A wavefront takes consecutive tokens of ONE KV head per step, so that its scores leave as
// one contiguous store (scores are [h][token] while the rows are [token][h]: writing one float per
// row in row order cost eight times the score bytes in partial-line writes). HBM-bound streaming.
//
// Window rule, scalar version: pass 1 gives every window row its log-sum-exp over the group's
// keys (one wavefront per row, lanes over keys); pass 2 gives every key the sum over rows of
// exp(logit - lse) (one thread per key, rows broadcast). The MFMA version lives in
// score_window_mfma.hip and is used when the layout allows it (bf16, head_dim 128).
#include "qp_internal.h"

namespace qp {

constexpr int NORM_UNROLL = 4;  // rows in flight per lane group: four independent 16-byte loads per lane

template <typename T, int D>
__global__ __launch_bounds__(256) void score_norm_kernel(const T* __restrict__ x, int n_g, int h_kv, float sign,
                                                         float* __restrict__ scores) {
  constexpr int PER = Elem<T>::kPer16B;
  constexpr int LPR = D / PER;             // lanes per row, power of two in 8..32
  constexpr int TW = 64 / LPR * NORM_UNROLL;  // tokens per wavefront item
  static_assert(LPR >= NORM_UNROLL && LPR <= 64, "row layout");
  const int lane = threadIdx.x & 63, sub = lane % LPR, lg = lane / LPR;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int n_waves = (gridDim.x * blockDim.x) >> 6;
  const int n_tb = (n_g + TW - 1) / TW;
  const long n_items = (long)n_tb * h_kv;  // item = (block of TW consecutive tokens, KV head); head fastest
  for (long item = wave; item < n_items; item += n_waves) {
    const int h = (int)(item % h_kv);
    const int t0 = (int)(item / h_kv) * TW + lg * NORM_UNROLL;  // this lane group's first token
    uint4 raw[NORM_UNROLL];
#pragma unroll
    for (int u = 0; u < NORM_UNROLL; ++u)
      raw[u] = t0 + u < n_g ? *(const uint4*)(x + ((size_t)(t0 + u) * h_kv + h) * D + sub * PER) : make_uint4(0, 0, 0, 0);
    float mine = 0.f;  // lane `sub` < NORM_UNROLL of the group ends up with token t0 + sub
#pragma unroll
    for (int u = 0; u < NORM_UNROLL; ++u) {
      float v[PER];
      widen16<T>(raw[u], v);
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < PER; ++e) ss = fmaf(v[e], v[e], ss);
#pragma unroll
      for (int o = LPR / 2; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
      if (sub == u) mine = ss;
    }
    // one store instruction per wavefront item: TW consecutive floats of scores[h][:]
    if (sub < NORM_UNROLL && t0 + sub < n_g) scores[(size_t)h * n_g + t0 + sub] = sign * sqrtf(mine) + 0.f;
  }
}

template <typename T, int D>
static void launch_norm(const void* x, int n_g, int h_kv, float sign, float* scores, hipStream_t s) {
  constexpr int TW = 64 / (D / Elem<T>::kPer16B) * NORM_UNROLL;
  const long items = (long)((n_g + TW - 1) / TW) * h_kv;
  long wgs = (items + 3) / 4;  // four wavefronts per workgroup, one item each
  if (wgs > 8192) wgs = 8192;  // wavefronts stride over the items beyond 32 workgroups per CU
  hipLaunchKernelGGL((score_norm_kernel<T, D>), dim3((unsigned)wgs), dim3(256), 0, s, (const T*)x, n_g, h_kv, sign, scores);
}

void launch_score_norm(const void* x, int dtype, int n_g, int h_kv, int d, float sign, float* scores,
                       hipStream_t s) {
  if (dtype == QP_F32) {
    if (d == 64) launch_norm<float, 64>(x, n_g, h_kv, sign, scores, s);
    else launch_norm<float, 128>(x, n_g, h_kv, sign, scores, s);
  } else {
    if (d == 64) launch_norm<bf16_t, 64>(x, n_g, h_kv, sign, scores, s);
    else launch_norm<bf16_t, 128>(x, n_g, h_kv, sign, scores, s);
  }
}

// ---------------------------------------------------------------------------------------------
// Softmax-free attention score: s[h][j] = scale * sum_{t, qh in head group h} Q_win[t, qh, :] . K_g[j, h, :]
//                                        = scale * qsum[h] . K_g[j, h, :],  qsum[h] = sum of the R*W window rows.
// Two launches: the window rows are summed once per KV head (f32, fixed order), then the keys are streamed like the
// norm rules (one KV head and consecutive tokens per wavefront, contiguous stores). HBM-bound.

template <typename T, int D>
__global__ __launch_bounds__(256) void window_qsum_kernel(const T* __restrict__ q_win, int w, int h_q, int h_kv,
                                                          float* __restrict__ qsum) {
  constexpr int PER = Elem<T>::kPer16B;
  constexpr int LPR = D / PER;       // lanes per row
  constexpr int RPI = 256 / LPR;     // rows per iteration of the workgroup
  __shared__ float part[RPI][D];
  const int h = blockIdx.x, r_heads = h_q / h_kv;
  const int sub = threadIdx.x % LPR, rg = threadIdx.x / LPR;
  float acc[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) acc[e] = 0.f;
  for (int row = rg; row < r_heads * w; row += RPI) {  // row = t * R + j, the memory order of the head group's rows
    const int t = row / r_heads, j = row - t * r_heads;
    const uint4 raw = *(const uint4*)(q_win + ((size_t)t * h_q + (size_t)h * r_heads + j) * D + sub * PER);
    float v[PER];
    widen16<T>(raw, v);
#pragma unroll
    for (int e = 0; e < PER; ++e) acc[e] += v[e];
  }
#pragma unroll
  for (int e = 0; e < PER; ++e) part[rg][sub * PER + e] = acc[e];
  __syncthreads();
  for (int e = threadIdx.x; e < D; e += 256) {
    float tot = 0.f;
    for (int g = 0; g < RPI; ++g) tot += part[g][e];
    qsum[(size_t)h * D + e] = tot;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void score_dot_kernel(const T* __restrict__ x, const float* __restrict__ qsum, int n_g,
                                                        int h_kv, float scale, float* __restrict__ scores) {
  constexpr int PER = Elem<T>::kPer16B;
  constexpr int LPR = D / PER;
  constexpr int TW = 64 / LPR * NORM_UNROLL;
  const int lane = threadIdx.x & 63, sub = lane % LPR, lg = lane / LPR;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int n_waves = (gridDim.x * blockDim.x) >> 6;
  const int n_tb = (n_g + TW - 1) / TW;
  const long n_items = (long)n_tb * h_kv;
  for (long item = wave; item < n_items; item += n_waves) {
    const int h = (int)(item % h_kv);
    const int t0 = (int)(item / h_kv) * TW + lg * NORM_UNROLL;
    float qs[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) qs[e] = qsum[(size_t)h * D + sub * PER + e];
    uint4 raw[NORM_UNROLL];
#pragma unroll
    for (int u = 0; u < NORM_UNROLL; ++u)
      raw[u] = t0 + u < n_g ? *(const uint4*)(x + ((size_t)(t0 + u) * h_kv + h) * D + sub * PER) : make_uint4(0, 0, 0, 0);
    float mine = 0.f;
#pragma unroll
    for (int u = 0; u < NORM_UNROLL; ++u) {
      float v[PER];
      widen16<T>(raw[u], v);
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < PER; ++e) dot = fmaf(v[e], qs[e], dot);
#pragma unroll
      for (int o = LPR / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
      if (sub == u) mine = dot;
    }
    if (sub < NORM_UNROLL && t0 + sub < n_g) scores[(size_t)h * n_g + t0 + sub] = scale * mine + 0.f;
  }
}

template <typename T, int D>
static void launch_logit(const WindowArgs& a, float scale, hipStream_t s) {
  constexpr int TW = 64 / (D / Elem<T>::kPer16B) * NORM_UNROLL;
  float* qsum = (float*)a.workspace;
  hipLaunchKernelGGL((window_qsum_kernel<T, D>), dim3(a.h_kv), dim3(256), 0, s, (const T*)a.q_win, a.w, a.h_q, a.h_kv, qsum);
  const long items = (long)((a.n_g + TW - 1) / TW) * a.h_kv;
  long wgs = (items + 3) / 4;
  if (wgs > 8192) wgs = 8192;
  hipLaunchKernelGGL((score_dot_kernel<T, D>), dim3((unsigned)wgs), dim3(256), 0, s, (const T*)a.k, qsum, a.n_g, a.h_kv,
                     scale, a.scores);
}

size_t window_logit_workspace_bytes(int h_kv, int d) { return ((size_t)h_kv * d * sizeof(float) + 255) / 256 * 256; }

// a.scale_log2 is not used here: `scale` is the softmax scale itself
void launch_score_window_logit(const WindowArgs& a, int dtype, float scale, hipStream_t s) {
  if (dtype == QP_F32) {
    if (a.d == 64) launch_logit<float, 64>(a, scale, s);
    else launch_logit<float, 128>(a, scale, s);
  } else {
    if (a.d == 64) launch_logit<bf16_t, 64>(a, scale, s);
    else launch_logit<bf16_t, 128>(a, scale, s);
  }
}

// Head-shared selection: scores[h][j] <- sum over h' of scores[h'][j], in head order, for every h.
__global__ __launch_bounds__(256) void share_heads_kernel(float* __restrict__ scores, int h_kv, int n_g) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n_g) return;
  float tot = 0.f;
  for (int h = 0; h < h_kv; ++h) tot += scores[(size_t)h * n_g + j];
  tot += 0.f;
  for (int h = 0; h < h_kv; ++h) scores[(size_t)h * n_g + j] = tot;
}

void launch_share_heads(float* scores, int h_kv, int n_g, hipStream_t s) {
  hipLaunchKernelGGL(share_heads_kernel, dim3((n_g + 255) / 256), dim3(256), 0, s, scores, h_kv, n_g);
}

// ---------------------------------------------------------------------------------------------
// Window rule, scalar version.

// lse2[qh][t] = log2( sum_j exp2(scale_log2 * q.k_j) ) over the group's n_g keys.
template <typename T, int D>
__global__ __launch_bounds__(256) void window_rowstats_kernel(WindowArgs a, float* __restrict__ lse2) {
  constexpr int WAVES = 4;
  constexpr int PER = Elem<T>::kPer16B;
  constexpr int CHUNKS = D / PER;
  __shared__ float q_lds[WAVES][D];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = blockIdx.x * WAVES + wave;
  const int qh = blockIdx.y;
  const int h = qh / (a.h_q / a.h_kv);
  const bool active = t < a.w;
  if (active) {
    const T* qrow = (const T*)a.q_win + ((size_t)t * a.h_q + qh) * D;
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
  const T* gk = (const T*)a.k + (size_t)h * D;
  const size_t gstride = (size_t)a.h_kv * D;
  for (int j = lane; j < a.n_g; j += 64) {
    const T* krow = gk + (size_t)j * gstride;
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
      l *= exp2f(m - s);
      m = s;
    }
    l += exp2f(s - m);
  }
  const float mw = wave_max(m);
  const float lw = wave_sum(l * exp2f(m - mw));
  if (lane == 0) lse2[(size_t)qh * a.w + t] = mw + log2f(lw);
}

// scores[h][j] = sum_{qh in head group h} sum_t exp2(scale_log2 * q.k_j - lse2[qh][t]).
template <typename T, int D>
__global__ __launch_bounds__(64) void window_colsum_kernel(WindowArgs a, const float* __restrict__ lse2) {
  constexpr int PER = Elem<T>::kPer16B;
  constexpr int CHUNKS = D / PER;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int h = blockIdx.y;
  if (j >= a.n_g) return;
  const int r = a.h_q / a.h_kv;
  float kv[D];
  const T* krow = (const T*)a.k + ((size_t)j * a.h_kv + h) * D;
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    uint4 raw = *(const uint4*)(krow + c * PER);
    widen16<T>(raw, kv + c * PER);
  }
  float total = 0.f;
  for (int qh = h * r; qh < (h + 1) * r; ++qh) {
    for (int t = 0; t < a.w; ++t) {
      const T* qrow = (const T*)a.q_win + ((size_t)t * a.h_q + qh) * D;  // uniform address: broadcast
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        uint4 raw = *(const uint4*)(qrow + c * PER);
        float qv[PER];
        widen16<T>(raw, qv);
#pragma unroll
        for (int e = 0; e < PER; ++e) s = fmaf(qv[e], kv[c * PER + e], s);
      }
      total += exp2f(s * a.scale_log2 - lse2[(size_t)qh * a.w + t]);
    }
  }
  a.scores[(size_t)h * a.n_g + j] = total;
}

size_t window_workspace_bytes(int h_q, int h_kv, int n_g, int w) {
  const size_t scalar = (size_t)h_q * w * sizeof(float);
  const size_t mfma = window_mfma_workspace_bytes(h_q, h_kv, n_g, w);
  return ((scalar > mfma ? scalar : mfma) + 255) / 256 * 256;
}

template <typename T, int D>
static void launch_window_t(const WindowArgs& a, hipStream_t s) {
  float* lse2 = (float*)a.workspace;
  hipLaunchKernelGGL((window_rowstats_kernel<T, D>), dim3((a.w + 3) / 4, a.h_q), dim3(256), 0, s, a, lse2);
  hipLaunchKernelGGL((window_colsum_kernel<T, D>), dim3((a.n_g + 63) / 64, a.h_kv), dim3(64), 0, s, a, lse2);
}

void launch_score_window(const WindowArgs& a, int dtype, hipStream_t s) {
  // the MFMA kernels form 32-bit byte offsets into the group's K
  if (window_mfma_supported(dtype, a.h_q, a.h_kv, a.d, a.w) && (long long)a.n_g * a.h_kv * (a.d * 2) < (1ll << 31)) {
    launch_score_window_mfma(a, s);
    return;
  }
  if (dtype == QP_F32) {
    if (a.d == 64) launch_window_t<float, 64>(a, s);
    else launch_window_t<float, 128>(a, s);
  } else {
    if (a.d == 64) launch_window_t<bf16_t, 64>(a, s);
    else launch_window_t<bf16_t, 128>(a, s);
  }
}

}  // namespace qp
