// The projections of the decoder layer for a handful of tokens (Sec. 2.1's last stage: decoding one token at a time
// through the layer, over the pruned cache), gfx950:
//   Y[m][n] = sum_k X[m][k] W[n][k],   m <= 2 tokens, W [N][K] bf16 weights ([out][in]), f32 accumulation,
// with the same three stores as the matrix-pipe kernel of gemm_bf16.hip (PLAIN: bias / residual; QKV_ROPE: bias,
// rotary embedding, scatter to Q / K / V; SWIGLU: SiLU(gate) * up; Appendix D.1 for the latter).
//
// With so few tokens the product is a stream of the weights: every weight byte is read once and meets m activations,
// so HBM is the bound and the matrix pipe has nothing to offer (a 256-row tile would hold one or two useful rows). The
// matrix-pipe kernel serves such calls by dealing the contraction to k chunks and summing their partial tiles in a
// second launch; this kernel does it in one launch and without partials in memory:
//   * a workgroup of 4 wavefronts owns 4 weight rows, chosen so that the values a store combines belong to the same
//     workgroup: 4 consecutive outputs (PLAIN), 2 dims of a head and their rotary partners (QKV_ROPE), 2 gate rows and
//     the up rows of the same outputs (SWIGLU);
//   * wavefront w walks the w-th quarter of k, 16 bytes per lane and row (a wavefront reads 1 KB runs of each row),
//     two such steps per loop trip with all of their loads issued before the first product, so that a wavefront has
//     8 KB of weights in flight and a compute unit (up to 32 wavefronts) well over the ~40 KB that 8 TB/s need at
//     ~2 us of latency; the activations (a few KB per token) come from L2 alongside;
//   * products are v_dot2_f32_bf16 (two multiply-adds per lane and instruction, f32 accumulation);
//   * the 64 lanes' sums are added by shuffles, the 4 wavefronts' sums meet in LDS and are added in wavefront order
//     (deterministic), and one lane per token applies the store.
#include "qp_internal.h"

namespace qp {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

constexpr int GV_WAVES = 4;
constexpr int GV_MAX_M = 2;  // tokens this kernel takes: every workgroup re-reads the activations, m / 4 of its weight bytes,
                             // and from 4 tokens on the tiled kernel with its split contraction is as fast or faster

__device__ __forceinline__ float dot8(const uint4& w, const uint4& x, float acc) {
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.x), __builtin_bit_cast(bf16x2, x.x), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.y), __builtin_bit_cast(bf16x2, x.y), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.z), __builtin_bit_cast(bf16x2, x.z), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.w), __builtin_bit_cast(bf16x2, x.w), acc, false);
  return acc;
}

// M: tokens computed (1 or 2)
template <int MODE, int M>
__global__ __launch_bounds__(GV_WAVES * 64) void gemv_bf16_kernel(GemmArgs a) {
  __shared__ float part[GV_WAVES][4][M];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int quad = blockIdx.x;  // < n / 4
  const int d_ff = a.n >> 1;
  // the 4 weight rows of this workgroup: y[0], y[1] and their partners y[2], y[3] in the store below
  int row[4];
  if (MODE == GEMM_QKV_ROPE) {
    const int head = quad >> 5, f0 = 2 * (quad & 31);
    row[0] = head * 128 + f0, row[1] = row[0] + 1, row[2] = row[0] + 64, row[3] = row[0] + 65;
  } else if (MODE == GEMM_SWIGLU) {
    row[0] = 2 * quad, row[1] = row[0] + 1, row[2] = d_ff + row[0], row[3] = d_ff + row[0] + 1;
  } else {
    row[0] = 4 * quad, row[1] = row[0] + 1, row[2] = row[0] + 2, row[3] = row[0] + 3;
  }
  const int chunks = a.k / 8, per_wave = chunks / GV_WAVES;  // k is a multiple of 64 (checked by the launcher)
  const int c_end = (wave + 1) * per_wave;
  const uint4* w[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = (const uint4*)((const bf16_t*)a.w + (size_t)row[e] * a.k);
  const uint4* x[M];
#pragma unroll
  for (int t = 0; t < M; ++t) x[t] = (const uint4*)((const bf16_t*)a.x + (size_t)min(t, a.m - 1) * a.k);

  float acc[4][M];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int t = 0; t < M; ++t) acc[e][t] = 0.f;
  const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
  for (int c = wave * per_wave + lane; c < c_end; c += 128) {
    const int c1 = c + 64;
    const bool has1 = c1 < c_end;
    uint4 w0[4], w1[4], x0[M], x1[M];
#pragma unroll
    for (int e = 0; e < 4; ++e) w0[e] = w[e][c];
#pragma unroll
    for (int t = 0; t < M; ++t) x0[t] = x[t][c];
#pragma unroll
    for (int e = 0; e < 4; ++e) w1[e] = has1 ? w[e][c1] : zero;
#pragma unroll
    for (int t = 0; t < M; ++t) x1[t] = has1 ? x[t][c1] : zero;
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int t = 0; t < M; ++t) acc[e][t] = dot8(w1[e], x1[t], dot8(w0[e], x0[t], acc[e][t]));
  }
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int t = 0; t < M; ++t) {
      const float s = wave_sum(acc[e][t]);
      if (lane == 0) part[wave][e][t] = s;
    }
  __syncthreads();
  const int t = threadIdx.x;
  if (t >= M || t >= a.m) return;
  float y[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) y[e] = ((part[0][e][t] + part[1][e][t]) + part[2][e][t]) + part[3][e][t];

  if (MODE == GEMM_PLAIN) {
    const int n = row[0];
    if (a.bias != nullptr) {
      const uint2 raw = *(const uint2*)((const bf16_t*)a.bias + n);
      y[0] += bf16lo_to_f32(raw.x), y[1] += bf16hi_to_f32(raw.x), y[2] += bf16lo_to_f32(raw.y), y[3] += bf16hi_to_f32(raw.y);
    }
    if (a.residual != nullptr) {
      const uint2 raw = *(const uint2*)((const bf16_t*)a.residual + (size_t)t * a.n + n);
      y[0] += bf16lo_to_f32(raw.x), y[1] += bf16hi_to_f32(raw.x), y[2] += bf16lo_to_f32(raw.y), y[3] += bf16hi_to_f32(raw.y);
    }
    uint2 pk;
    pk.x = (uint32_t)f32_to_bf16_rne(y[0]) | ((uint32_t)f32_to_bf16_rne(y[1]) << 16);
    pk.y = (uint32_t)f32_to_bf16_rne(y[2]) | ((uint32_t)f32_to_bf16_rne(y[3]) << 16);
    *(uint2*)((bf16_t*)a.out + (size_t)t * a.n + n) = pk;
  } else if (MODE == GEMM_QKV_ROPE) {
    const int head = quad >> 5, f0 = 2 * (quad & 31);  // f0: first of 2 rotary frequencies
    const bf16_t* bias = (const bf16_t*)a.bias + (size_t)head * 128;
    const uint32_t b0 = *(const uint32_t*)(bias + f0), b1 = *(const uint32_t*)(bias + 64 + f0);
    float lo[2] = {y[0] + bf16lo_to_f32(b0), y[1] + bf16hi_to_f32(b0)};
    float hi[2] = {y[2] + bf16lo_to_f32(b1), y[3] + bf16hi_to_f32(b1)};
    bf16_t* dst;
    int heads_dst, head_dst;
    if (head < a.h_q) dst = (bf16_t*)a.q, heads_dst = a.h_q, head_dst = head;
    else if (head < a.h_q + a.h_kv) dst = (bf16_t*)a.k_out, heads_dst = a.h_kv, head_dst = head - a.h_q;
    else dst = (bf16_t*)a.v_out, heads_dst = a.h_kv, head_dst = head - a.h_q - a.h_kv;
    if (head < a.h_q + a.h_kv) {
      const float4 cs = *(const float4*)(a.cos_sin + ((size_t)t * 64 + f0) * 2);  // (cos, sin) of f0 and f0 + 1
      const float c[2] = {cs.x, cs.z}, sn[2] = {cs.y, cs.w};
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const float x0 = lo[e], x1 = hi[e];
        lo[e] = x0 * c[e] - x1 * sn[e];
        hi[e] = x1 * c[e] + x0 * sn[e];
      }
    }
    bf16_t* out_row = dst + ((size_t)t * heads_dst + head_dst) * 128;
    *(uint32_t*)(out_row + f0) = (uint32_t)f32_to_bf16_rne(lo[0]) | ((uint32_t)f32_to_bf16_rne(lo[1]) << 16);
    *(uint32_t*)(out_row + 64 + f0) = (uint32_t)f32_to_bf16_rne(hi[0]) | ((uint32_t)f32_to_bf16_rne(hi[1]) << 16);
  } else {  // GEMM_SWIGLU: y[0], y[1] gate and y[2], y[3] up of outputs row[0], row[0] + 1
    const float o0 = y[0] / (1.f + __expf(-y[0])) * y[2], o1 = y[1] / (1.f + __expf(-y[1])) * y[3];
    *(uint32_t*)((bf16_t*)a.out + (size_t)t * d_ff + row[0]) =
        (uint32_t)f32_to_bf16_rne(o0) | ((uint32_t)f32_to_bf16_rne(o1) << 16);
  }
}

// The shapes gemm_supported admits all fit: k is a multiple of 64 (a wavefront's quarter of it a whole number of
// 16-byte chunks), n a multiple of 8 (PLAIN), of 128 per head (QKV_ROPE) or of 256 (SWIGLU), hence of 4.
bool gemv_applies(const GemmArgs& a) { return a.m <= GV_MAX_M; }

template <int MODE>
static hipError_t launch_gemv_mode(const GemmArgs& a, hipStream_t s) {
  const dim3 grid((unsigned)(a.n / 4)), block(GV_WAVES * 64);
  if (a.m == 1) hipLaunchKernelGGL((gemv_bf16_kernel<MODE, 1>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((gemv_bf16_kernel<MODE, 2>), grid, block, 0, s, a);
  return hipSuccess;
}

hipError_t launch_gemv_bf16(const GemmArgs& a, int mode, hipStream_t s) {
  if (!gemv_applies(a) || !gemm_supported(a, mode)) return hipErrorInvalidValue;
  switch (mode) {
    case GEMM_PLAIN: return launch_gemv_mode<GEMM_PLAIN>(a, s);
    case GEMM_QKV_ROPE: return launch_gemv_mode<GEMM_QKV_ROPE>(a, s);
    case GEMM_SWIGLU: return launch_gemv_mode<GEMM_SWIGLU>(a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace qp
