// "Attention Scores" importance rule (third function under Eq. 2, Sec. 3.2) on bf16 MFMA, head_dim 128.
//
//   s[h][j] = sum over the R query heads of KV head h and the W window rows t of
//             softmax_j( scale * Q_win[t, qh, :] . K_g[j, h, :] ),   softmax over the group's N_g keys.
//
// The R*W window rows of a KV head are stacked as row = t*R + j (their memory order in
// Q_win[t][h*R + j][:]). The work is a (R*W) x N_g x 128 contraction done twice; the whole problem is
// a few MB and ~1 % of the attention flops, so the kernels are shaped for latency, not for the roof:
//   pass 1   one wavefront per (32 rows, chunk of 64..1024 keys, 64 at a time): Q and both K blocks are requested
//            up front (24 loads in flight), S^T = K . Q^T, a lane holds one row, so the row max and sum of
//            exponentials are in-register reductions; one (m, l) partial per (row, chunk).
//   pass 2   a workgroup first merges the partials into lse[row] in LDS (padded rows get +inf = weight 0);
//            it owns 128 keys (32 per wavefront, K fragments in registers) and stages the head's
//            window rows in LDS (direct global -> LDS loads, XOR-swizzled 16-byte chunks, up to 512 rows
//            at a time); per 32-row block S = Q . K^T (a lane holds one key, rows in registers),
//            p = exp2(c*s - lse[row]), and the column sum over all rows is an in-register sum plus one
//            exchange between lane l and l+32.
// No atomics: results are deterministic.
#include "qp_internal.h"

namespace qp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int WIN_D = 128;
constexpr int WIN_KC = 64;          // keys per pass-1 task
constexpr int WIN_MAX_ROWS = 8192;  // R*W rows (padded to 32) this path takes
constexpr int WIN_CH = 512;         // window rows staged in LDS at a time in pass 2 (128 KB)
constexpr int WIN_P2_KEYS = 128;    // keys per pass-2 workgroup

__host__ __device__ inline int win_rows_padded(int h_q, int h_kv, int w) { return ((h_q / h_kv) * w + 31) / 32 * 32; }

// partial[h][kc][row] = (m * c2, l): max of the scaled logits over chunk kc and sum of exp2 around it. A chunk is
// kc_sub sub-chunks of 64 keys walked by one wavefront with the Q fragments kept in registers (kc_sub = 1 for
// small groups: most parallelism, least latency; larger for long groups, so that pass 2 merges at most 32
// partials per row and Q is fetched once per chunk).
__global__ __launch_bounds__(256) void window_pass1_kernel(WindowArgs a, float2* __restrict__ partial, int kc_sub) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int h = blockIdx.y;
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = r_heads * a.w;
  const int n_rows_pad = win_rows_padded(a.h_q, a.h_kv, a.w);
  const int n_rbk = n_rows_pad / 32;
  const int chunk_keys = WIN_KC * kc_sub;
  const int n_kc = (a.n_g + chunk_keys - 1) / chunk_keys;
  const int task = blockIdx.x * 4 + wave;
  if (task >= n_rbk * n_kc) return;
  const int kc = task / n_rbk, rbk = task - kc * n_rbk;

  const int row = rbk * 32 + l32;
  const int rowc = min(row, n_rows - 1);
  const int t = rowc / r_heads, j = rowc - t * r_heads;
  const bf16_t* qrow = (const bf16_t*)a.q_win + ((size_t)t * a.h_q + (size_t)h * r_heads + j) * WIN_D;
  const bf16_t* gk = (const bf16_t*)a.k + (size_t)h * WIN_D;
  const size_t gstride = (size_t)a.h_kv * WIN_D;
  const float c2 = a.scale_log2;
  // Q and the first sub-chunk's K: all 24 fragment loads are issued before the first use
  u32x4 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) qf[s] = *(const u32x4*)(qrow + 16 * s + 8 * g);
  float m_run = -INFINITY, l_run = 0.f;  // over the sub-chunks so far (m in scaled log2 units)
  for (int sub = 0; sub < kc_sub; ++sub) {
    const int k0 = kc * chunk_keys + sub * WIN_KC;
    if (k0 >= a.n_g) break;  // the chunk's first sub-chunk always exists
    u32x4 kf[2][8];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const bf16_t* krow = gk + (size_t)min(k0 + 32 * b + l32, a.n_g - 1) * gstride;
#pragma unroll
      for (int s = 0; s < 8; ++s) kf[b][s] = *(const u32x4*)(krow + 16 * s + 8 * g);
    }
    f32x16 st[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
      for (int r = 0; r < 16; ++r) st[b][r] = 0.f;
#pragma unroll
      for (int s = 0; s < 8; ++s)
        st[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[b][s]),
                                                        __builtin_bit_cast(bf16x8, qf[s]), st[b], 0, 0, 0);
    }
    if (k0 + WIN_KC > a.n_g) {  // ragged last sub-chunk: its first key exists, the rest may not
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (k0 + 32 * b + 8 * (r >> 2) + 4 * g + (r & 3) >= a.n_g) st[b][r] = -INFINITY;
    }
    float mx = st[0][0];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[b][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float mc = mx * c2;  // finite: key k0 exists
    float psum = 0.f;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) psum += __builtin_amdgcn_exp2f(fmaf(st[b][r], c2, -mc));
    psum += __shfl_xor(psum, 32, 64);
    const float m_new = fmaxf(m_run, mc);
    l_run = l_run * __builtin_amdgcn_exp2f(m_run - m_new) + psum * __builtin_amdgcn_exp2f(mc - m_new);
    m_run = m_new;
  }
  if (g == 0) partial[((size_t)h * n_kc + kc) * n_rows_pad + row] = make_float2(m_run, l_run);
}

__global__ __launch_bounds__(256) void window_pass2_kernel(WindowArgs a, const float2* __restrict__ partial, int kc_sub) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [ch_rows x 256 B of Q][n_rows_pad floats of lse]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int h = blockIdx.y;
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = r_heads * a.w;
  const int n_rows_pad = win_rows_padded(a.h_q, a.h_kv, a.w);
  const int ch_rows = min(n_rows_pad, WIN_CH);
  float* lse2 = (float*)(smem + (size_t)ch_rows * 256);
  const unsigned char* qbase = (const unsigned char*)a.q_win + (size_t)h * r_heads * (WIN_D * 2);
  const unsigned q_tok_stride = (unsigned)a.h_q * (WIN_D * 2);
  // stage window rows [c0_, c0_ + rows_): one load instruction moves 4 rows; lane -> (row, LDS position)
#define QP_STAGE_ROWS(c0_, rows_)                                                                          \
  for (int i = wave; i < (rows_) / 4; i += 4) {                                                            \
    const int rl = 4 * i + (lane >> 4);           /* row inside the chunk */                               \
    const int rowc = min((c0_) + rl, n_rows - 1); /* padded rows re-read the last row; their weight is 0 */ \
    const int t = rowc / r_heads, j = rowc - t * r_heads;                                                  \
    const unsigned off = (unsigned)t * q_tok_stride + (unsigned)j * (WIN_D * 2) +                          \
                         (unsigned)((((lane & 15) ^ (rl & 15))) << 4);                                     \
    lds_dma16(qbase, off, smem + (size_t)i * 1024);                                                        \
  }
  // The first chunk of rows is requested before anything else: it lands while the partials are merged.
  QP_STAGE_ROWS(0, min(ch_rows, n_rows_pad))

  // this wavefront's 32 keys as the B operand (K^T), held in registers for the whole kernel
  const int k0 = blockIdx.x * WIN_P2_KEYS + wave * 32;
  const bool wave_live = k0 < a.n_g;
  const bf16_t* krow = (const bf16_t*)a.k + ((size_t)min(k0 + l32, a.n_g - 1) * a.h_kv + h) * WIN_D;
  bf16x8 kf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) kf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(krow + 16 * s + 8 * g));

  // lse2[row] = log2 sum_j exp2(c2 * s_j), merged from the chunk partials (every workgroup repeats this small
  // reduction: it is cheaper than a launch); padded rows get +inf, i.e. weight 0 below. The partials of a row
  // are read eight at a time so that the loads overlap.
  {
    const int n_kc = (a.n_g + WIN_KC * kc_sub - 1) / (WIN_KC * kc_sub);
    for (int r = tid; r < n_rows_pad; r += 256) {
      float v = INFINITY;
      if (r < n_rows) {
        const float2* p = partial + (size_t)h * n_kc * n_rows_pad + r;
        float m = -INFINITY, l = 0.f;
        for (int kc0 = 0; kc0 < n_kc; kc0 += 8) {
          float2 e[8];
#pragma unroll
          for (int u = 0; u < 8; ++u)
            e[u] = kc0 + u < n_kc ? p[(size_t)(kc0 + u) * n_rows_pad] : make_float2(-INFINITY, 0.f);
          float mb = e[0].x;
#pragma unroll
          for (int u = 1; u < 8; ++u) mb = fmaxf(mb, e[u].x);
          const float m_new = fmaxf(m, mb);  // finite: chunk kc0 exists
          l *= __builtin_amdgcn_exp2f(m - m_new);
#pragma unroll
          for (int u = 0; u < 8; ++u) l += e[u].y * __builtin_amdgcn_exp2f(e[u].x - m_new);
          m = m_new;
        }
        v = m + log2f(l);
      }
      lse2[r] = v;
    }
  }

  const float c2 = a.scale_log2;
  float colsum = 0.f;
  int a_addr[8];  // A fragment (Q rows) of d-step s: row l32 of the block, chunk 2s+g at position (2s+g) ^ (l32 & 15)
#pragma unroll
  for (int s = 0; s < 8; ++s) a_addr[s] = l32 * 256 + (((2 * s + g) ^ (l32 & 15)) << 4);

  for (int c0 = 0; c0 < n_rows_pad; c0 += ch_rows) {
    const int rows_here = min(ch_rows, n_rows_pad - c0);
    if (c0 > 0) QP_STAGE_ROWS(c0, rows_here)
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): staged rows (and, the first time, K fragments and partials)
    __syncthreads();
    if (wave_live) {
      for (int rbk = 0; rbk < rows_here / 32; ++rbk) {
        const unsigned char* qt = smem + (size_t)rbk * 32 * 256;
        u32x4 af[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) af[s] = *(const u32x4*)(qt + a_addr[s]);
        f32x16 sc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s)
          sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[s]), kf[s], sc, 0, 0, 0);
        // register r holds row c0 + rbk*32 + 8*(r/4) + 4*g + r%4 for this lane's key
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const float4 ls = *(const float4*)&lse2[c0 + rbk * 32 + 8 * q4 + 4 * g];
          colsum += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 0], c2, -ls.x));
          colsum += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 1], c2, -ls.y));
          colsum += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 2], c2, -ls.z));
          colsum += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 3], c2, -ls.w));
        }
      }
    }
    __syncthreads();  // before the next chunk overwrites the staged rows
  }
#undef QP_STAGE_ROWS
  colsum += __shfl_xor(colsum, 32, 64);
  if (wave_live && g == 0 && k0 + l32 < a.n_g) a.scores[(size_t)h * a.n_g + k0 + l32] = colsum;
}

bool window_mfma_supported(int dtype, int h_q, int h_kv, int d, int w) {
  const long long q_bytes = (long long)w * h_q * d * 2;  // 32-bit byte offsets into the window tensor
  return dtype == QP_BF16 && d == WIN_D && win_rows_padded(h_q, h_kv, w) <= WIN_MAX_ROWS && q_bytes < (1ll << 31);
}

size_t window_mfma_workspace_bytes(int h_q, int h_kv, int n_g, int w) {
  const size_t n_kc = (n_g + WIN_KC - 1) / WIN_KC;
  const size_t rows = win_rows_padded(h_q, h_kv, w);
  return (size_t)h_kv * n_kc * rows * sizeof(float2);
}

void launch_score_window_mfma(const WindowArgs& a, hipStream_t s) {
  const int rows = win_rows_padded(a.h_q, a.h_kv, a.w);
  const int n_rbk = rows / 32;
  int kc_sub = 1;  // sub-chunks of 64 keys per pass-1 chunk: at most 32 chunks per row for pass 2 to merge
  while ((a.n_g + WIN_KC * kc_sub - 1) / (WIN_KC * kc_sub) > 32) kc_sub *= 2;
  const int n_kc = (a.n_g + WIN_KC * kc_sub - 1) / (WIN_KC * kc_sub);
  float2* partial = (float2*)a.workspace;  // sized for kc_sub = 1
  const size_t lds2 = (size_t)(rows < WIN_CH ? rows : WIN_CH) * 256 + (size_t)rows * sizeof(float);
  static bool attr_set[QP_MAX_DEVICES] = {};
  const int dev = current_device();
  if (dev < 0 || !attr_set[dev]) {
    (void)hipFuncSetAttribute((const void*)window_pass2_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                              WIN_CH * 256 + WIN_MAX_ROWS * (int)sizeof(float));
    if (dev >= 0) attr_set[dev] = true;
  }
  hipLaunchKernelGGL(window_pass1_kernel, dim3((n_rbk * n_kc + 3) / 4, a.h_kv), dim3(256), 0, s, a, partial, kc_sub);
  hipLaunchKernelGGL(window_pass2_kernel, dim3((a.n_g + WIN_P2_KEYS - 1) / WIN_P2_KEYS, a.h_kv), dim3(256), lds2, s, a,
                     partial, kc_sub);
}

}  // namespace qp
