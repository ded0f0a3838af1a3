// "Attention Scores" importance rule (third function under Eq. 2, Sec. 3.2) on bf16 MFMA, head_dim 128.
//
//   s[h][j] = sum over the R query heads of KV head h and the W window rows t of
//             softmax_j( scale * Q_win[t, qh, :] . K_g[j, h, :] ),   softmax over the group's N_g keys.
//
// The R*W window rows of a KV head are stacked as row = t*R + j (their memory order in
// Q_win[t][h*R + j][:]). The work is a (R*W) x N_g x 128 contraction done twice:
//   pass 1  S^T = K . Q^T per (32-row block, chunk of WIN_KC keys): a lane holds one row, so the
//           chunk's row max and sum of exponentials are in-register reductions; one (m, l) partial
//           per (row, chunk) goes to the workspace.
//   pass 2  per 32-key block: the partials are merged into lse[row] in LDS, then S = Q . K^T
//           (a lane holds one key, rows in registers), p = exp2(c*s - lse[row]) and the column
//           sum over all rows is an in-register sum plus one exchange between lane l and l+32.
// Operands come straight from global memory / L2 (each is used by one wavefront only; the
// whole problem is a few MB and ~1% of the attention flops). No atomics: results are
// deterministic.
#include "qp_internal.h"

namespace qp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int WIN_D = 128;
constexpr int WIN_KC = 256;        // keys per pass-1 task
constexpr int WIN_MAX_ROWS = 4096; // R*W rows (padded to 32) the LDS table of pass 2 holds

__host__ __device__ inline int win_rows_padded(int h_q, int h_kv, int w) { return ((h_q / h_kv) * w + 31) / 32 * 32; }

// partial[h][kc][row] = (m * c2, l): max of the scaled logits over the chunk and sum of exp2 around it.
__global__ __launch_bounds__(256) void window_pass1_kernel(WindowArgs a, float2* __restrict__ partial) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int h = blockIdx.y;
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = r_heads * a.w;
  const int n_rows_pad = win_rows_padded(a.h_q, a.h_kv, a.w);
  const int n_rbk = n_rows_pad / 32;
  const int n_kc = (a.n_g + WIN_KC - 1) / WIN_KC;
  const int task = blockIdx.x * 4 + wave;
  if (task >= n_rbk * n_kc) return;
  const int kc = task / n_rbk, rbk = task - kc * n_rbk;

  const int row = rbk * 32 + l32;
  const int rowc = min(row, n_rows - 1);
  const int t = rowc / r_heads, j = rowc - t * r_heads;
  const bf16_t* qrow = (const bf16_t*)a.q_win + ((size_t)t * a.h_q + (size_t)h * r_heads + j) * WIN_D;
  bf16x8 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) qf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + 16 * s + 8 * g));

  const bf16_t* gk = (const bf16_t*)a.k + (size_t)h * WIN_D;
  const size_t gstride = (size_t)a.h_kv * WIN_D;
  const float c2 = a.scale_log2;
  float m_run = -INFINITY, l_run = 0.f;
  const int key_end = min((kc + 1) * WIN_KC, a.n_g);
  for (int k0 = kc * WIN_KC; k0 < key_end; k0 += 32) {
    const int key = min(k0 + l32, a.n_g - 1);
    const bf16_t* krow = gk + (size_t)key * gstride;
    f32x16 st;
#pragma unroll
    for (int r = 0; r < 16; ++r) st[r] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const u32x4 raw = *(const u32x4*)(krow + 16 * s + 8 * g);
      st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), qf[s], st, 0, 0, 0);
    }
    if (k0 + 32 > a.n_g) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (k0 + 8 * (r >> 2) + 4 * g + (r & 3) >= a.n_g) st[r] = -INFINITY;
    }
    float mx = st[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, st[r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);   // finite: the first key of every chunk exists
    const float mc = m_new * c2;
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) psum += __builtin_amdgcn_exp2f(fmaf(st[r], c2, -mc));
    l_run = l_run * __builtin_amdgcn_exp2f((m_run - m_new) * c2) + psum;
    m_run = m_new;
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (g == 0) partial[((size_t)h * n_kc + kc) * n_rows_pad + row] = make_float2(m_run * c2, l_tot);
}

__global__ __launch_bounds__(256) void window_pass2_kernel(WindowArgs a, const float2* __restrict__ partial) {
  __shared__ __attribute__((aligned(16))) float lse2[WIN_MAX_ROWS];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int h = blockIdx.y;
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = r_heads * a.w;
  const int n_rows_pad = win_rows_padded(a.h_q, a.h_kv, a.w);
  const int n_kc = (a.n_g + WIN_KC - 1) / WIN_KC;

  // merge the chunk partials: lse2[row] = log2 sum_j exp2(c2 * s_j); padded rows get +inf (weight 0)
  for (int row = tid; row < n_rows_pad; row += 256) {
    float v = INFINITY;
    if (row < n_rows) {
      const float2* p = partial + (size_t)h * n_kc * n_rows_pad + row;
      float m = -INFINITY;
      for (int kc = 0; kc < n_kc; ++kc) m = fmaxf(m, p[(size_t)kc * n_rows_pad].x);
      float l = 0.f;
      for (int kc = 0; kc < n_kc; ++kc) {
        const float2 e = p[(size_t)kc * n_rows_pad];
        l += e.y * __builtin_amdgcn_exp2f(e.x - m);
      }
      v = m + log2f(l);
    }
    lse2[row] = v;
  }
  __syncthreads();

  const int k0 = (blockIdx.x * 4 + wave) * 32;
  if (k0 >= a.n_g) return;
  const int key = min(k0 + l32, a.n_g - 1);
  const bf16_t* krow = (const bf16_t*)a.k + ((size_t)key * a.h_kv + h) * WIN_D;
  bf16x8 kf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) kf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(krow + 16 * s + 8 * g));

  const float c2 = a.scale_log2;
  float colsum = 0.f;
  const bf16_t* qbase = (const bf16_t*)a.q_win + (size_t)h * r_heads * WIN_D;
  for (int rbk = 0; rbk < n_rows_pad / 32; ++rbk) {
    const int rowc = min(rbk * 32 + l32, n_rows - 1);
    const int t = rowc / r_heads, j = rowc - t * r_heads;
    const bf16_t* qrow = qbase + ((size_t)t * a.h_q + j) * WIN_D;
    f32x16 sc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const u32x4 raw = *(const u32x4*)(qrow + 16 * s + 8 * g);
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), kf[s], sc, 0, 0, 0);
    }
    // register r holds row rbk*32 + 8*(r/4) + 4*g + r%4 for this lane's key
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const float4 ls = *(const float4*)&lse2[rbk * 32 + 8 * q4 + 4 * g];
      colsum += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 0], c2, -ls.x));
      colsum += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 1], c2, -ls.y));
      colsum += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 2], c2, -ls.z));
      colsum += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 3], c2, -ls.w));
    }
  }
  colsum += __shfl_xor(colsum, 32, 64);
  if (g == 0 && k0 + l32 < a.n_g) a.scores[(size_t)h * a.n_g + k0 + l32] = colsum;
}

bool window_mfma_supported(int dtype, int h_q, int h_kv, int d, int w) {
  return dtype == QP_BF16 && d == WIN_D && win_rows_padded(h_q, h_kv, w) <= WIN_MAX_ROWS;
}

size_t window_mfma_workspace_bytes(int h_q, int h_kv, int n_g, int w) {
  const size_t n_kc = (n_g + WIN_KC - 1) / WIN_KC;
  return (size_t)h_kv * n_kc * win_rows_padded(h_q, h_kv, w) * sizeof(float2);
}

void launch_score_window_mfma(const WindowArgs& a, hipStream_t s) {
  const int n_rbk = win_rows_padded(a.h_q, a.h_kv, a.w) / 32;
  const int n_kc = (a.n_g + WIN_KC - 1) / WIN_KC;
  float2* partial = (float2*)a.workspace;
  hipLaunchKernelGGL(window_pass1_kernel, dim3((n_rbk * n_kc + 3) / 4, a.h_kv), dim3(256), 0, s, a, partial);
  hipLaunchKernelGGL(window_pass2_kernel, dim3((a.n_g + 127) / 128, a.h_kv), dim3(256), 0, s, a, partial);
}

}  // namespace qp
