// "Attention Scores" importance rule (third function under Eq. 2, Sec. 3.2) on bf16 MFMA, head_dim 128.
//
//   s[h][j] = sum over the R query heads of KV head h and the W window rows t of
//             softmax_j( scale * Q_win[t, qh, :] . K_g[j, h, :] ),   softmax over the group's N_g keys.
//
// The R*W window rows of a KV head are stacked as row = t*R + j (their memory order in
// Q_win[t][h*R + j][:]). The work is a (R*W) x N_g x 128 contraction done twice: the row normalisers need all
// keys before any column sum can be formed.
//   pass 1   log-sum-exp partials per (row, key chunk)
//   pass 2   column sums of exp2(c * s - lse[row])
// Both passes are one kernel template with the same decomposition: a workgroup of 8 wavefronts owns one
// KV head's chunk of 64..256 keys, stages it ONCE in LDS (direct global -> LDS loads, XOR-swizzled 16-byte
// chunks as in the attention kernel), and its wavefronts share the head's row blocks of 32 window rows
// (wavefront w takes blocks w, w+8, ...), whose fragments come straight from global memory into registers:
// the window tensor is a few hundred KB and lives in L2. So a group's K is read once per pass and the window once
// per key chunk from L2. Workgroup ids are dealt to (head, chunk) the same way in both passes and so that one
// head's workgroups share XCDs (ids go round-robin over the 8 XCDs, each with its own L2): the second pass finds
// its key chunk in the L2 that the first pass filled, and an L2 holds one head's window rows instead of all.
//   pass 1   S^T = K . Q^T per 64 keys: a lane holds one row, so the running row max / sum of exponentials over
//            the chunk are in-register reductions plus one exchange between lane l and l+32.
//   pass 2   every wavefront first merges its rows' partials into lse[row] (lanes over rows, all loads of a
//            batch in flight together); S = Q . K^T per 32 keys: a lane holds one key and registers hold rows, so
//            the sum over rows is in-register; per-wavefront column sums meet in LDS and are added in wavefront
//            order.
// No atomics: results are deterministic.
#include "qp_internal.h"

namespace qp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int WIN_D = 128;
constexpr int WIN_NW = 8;           // wavefronts per workgroup
constexpr int WIN_NT = WIN_NW * 64;
constexpr int WIN_KC_MIN = 64;      // keys per workgroup: a multiple of 64 between these two
constexpr int WIN_KC_MAX = 256;
constexpr int WIN_MAX_KB = WIN_KC_MAX / 32;
constexpr int WIN_MAX_ROWS = 8192;  // R*W rows (padded to 32) this path takes
constexpr int WIN_WANT_CHUNKS = 32; // key chunks per head aimed for (pass 2 merges that many partials per row)

__host__ __device__ inline int win_rows_padded(int h_q, int h_kv, int w) { return ((h_q / h_kv) * w + 31) / 32 * 32; }

// Keys per workgroup: about n_g / 32, a multiple of 64 in [64, 256] (host and device agree through the argument).
static int win_chunk_keys(int n_g) {
  int kc = ((n_g + WIN_WANT_CHUNKS - 1) / WIN_WANT_CHUNKS + 63) / 64 * 64;
  return kc < WIN_KC_MIN ? WIN_KC_MIN : (kc > WIN_KC_MAX ? WIN_KC_MAX : kc);
}

// PASS 1: partial[h][kc][row] = (m, l): max of the scaled logits (log2 units) over key chunk kc and the sum of
//         exp2 around it.
// PASS 2: scores[h][j] for the chunk's keys from the merged partials.
template <int PASS>
__global__ __launch_bounds__(WIN_NT) void window_kernel(WindowArgs a, float2* __restrict__ partial, int kc_keys, int n_kc) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [kc_keys x 256 B of K][pass 2: lse, column sums]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g = lane >> 5;
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = r_heads * a.w;
  const int n_rows_pad = win_rows_padded(a.h_q, a.h_kv, a.w);
  const int n_rbk = n_rows_pad / 32;
  // workgroup id -> (KV head, key chunk), one head's workgroups on the same XCDs
  int h, kc;
  {
    const int wg = blockIdx.x, xcd = wg & 7, idx = wg >> 3;
    if (8 % a.h_kv == 0) {
      const int per = 8 / a.h_kv;
      h = xcd / per;
      kc = idx * per + (xcd % per);
    } else if (a.h_kv % 8 == 0) {
      const int hp = a.h_kv / 8;
      h = (idx % hp) * 8 + xcd;
      kc = idx / hp;
    } else {
      h = wg % a.h_kv;
      kc = wg / a.h_kv;
    }
  }
  if (kc >= n_kc) return;  // padding workgroups of the XCD mapping (whole workgroup, before any barrier)
  const int k0 = kc * kc_keys;

  // stage the chunk's keys: one load instruction moves 4 key rows; chunk c of key k lands at position c ^ (k & 15)
  {
    const unsigned char* gk = (const unsigned char*)a.k + (size_t)h * (WIN_D * 2);
    const unsigned gstride = (unsigned)a.h_kv * (WIN_D * 2);
    for (int i = wave; i < kc_keys / 4; i += WIN_NW) {
      const int kl = 4 * i + (lane >> 4);
      const unsigned row_b = __umul24((unsigned)min(k0 + kl, a.n_g - 1), gstride);  // keys past the end are masked below
      lds_dma16(gk, row_b + (unsigned)((((lane & 15) ^ (kl & 15))) << 4), smem + (size_t)i * 1024);
    }
  }
  float* lse_w = (float*)(smem + (size_t)kc_keys * 256) + wave * 32;  // pass 2: this wavefront's 32 row normalisers
  float* red = (float*)(smem + (size_t)kc_keys * 256) + WIN_NW * 32;  // pass 2: [wavefront][key] column sums

  int k_addr[8];  // K fragment of d-step s: key l32 of a 32-key block, chunk 2s+g at position (2s+g) ^ (l32 & 15)
#pragma unroll
  for (int s = 0; s < 8; ++s) k_addr[s] = l32 * 256 + (((2 * s + g) ^ (l32 & 15)) << 4);
  const float c2 = a.scale_log2;
  const int n_kb = kc_keys / 32;
  float colsum[WIN_MAX_KB];
#pragma unroll
  for (int kb = 0; kb < WIN_MAX_KB; ++kb) colsum[kb] = 0.f;

  bool staged = false;
  for (int rbk = wave; rbk < n_rbk; rbk += WIN_NW) {
    // this block's window rows: lane l32 holds d = 16 s + 8 g .. + 7 of row rbk*32 + l32 (padded rows repeat the last)
    const int row = rbk * 32 + l32;
    const int rowc = min(row, n_rows - 1);
    const int t = rowc / r_heads, j = rowc - t * r_heads;
    const bf16_t* qrow = (const bf16_t*)a.q_win + ((size_t)t * a.h_q + (size_t)h * r_heads + j) * WIN_D;
    bf16x8 qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + 16 * s + 8 * g));
    if (PASS == 2) {
      // lse[row] = log2 sum_j exp2(c2 s_j) from the chunk partials; the two half-wavefronts split the chunks of a row
      float v = INFINITY;  // padded rows: weight 0
      const float2* p = partial + (size_t)h * n_kc * n_rows_pad + rowc;
      float m = -INFINITY, l = 0.f;
      for (int c0 = g; c0 < n_kc; c0 += 16) {
        float2 e[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          e[u] = c0 + 2 * u < n_kc ? p[(size_t)(c0 + 2 * u) * n_rows_pad] : make_float2(-INFINITY, 0.f);
        float mb = e[0].x;
#pragma unroll
        for (int u = 1; u < 8; ++u) mb = fmaxf(mb, e[u].x);
        const float m_new = fmaxf(m, mb);  // finite: chunk c0 exists
        l *= __builtin_amdgcn_exp2f(m - m_new);
#pragma unroll
        for (int u = 0; u < 8; ++u) l += e[u].y * __builtin_amdgcn_exp2f(e[u].x - m_new);
        m = m_new;
      }
      // combine the halves (a half without chunks holds m = -inf, l = 0: n_kc == 1)
      const float mo = __shfl_xor(m, 32, 64), lo = __shfl_xor(l, 32, 64);
      const float mm = fmaxf(m, mo);
      const float ll = l * __builtin_amdgcn_exp2f(m - mm) + lo * __builtin_amdgcn_exp2f(mo - mm);
      if (row < n_rows) v = mm + log2f(ll);
      if (g == 0) lse_w[l32] = v;  // read back below by all lanes of this wavefront (LDS keeps a wavefront's order)
    }
    if (!staged) {  // the first row block's loads overlap the staging of the keys
      __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
      __syncthreads();
      staged = true;
    }
    if (PASS == 1) {
      float m_run = -INFINITY, l_run = 0.f;
      for (int kb2 = 0; kb2 < n_kb / 2; ++kb2) {
        const int kbase = k0 + kb2 * 64;
        if (kbase >= a.n_g) break;  // wave-uniform: nothing of this and the later sub-blocks exists
        const unsigned char* kt = smem + (size_t)kb2 * 64 * 256;
        u32x4 kf[2][8];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int s = 0; s < 8; ++s) kf[b][s] = *(const u32x4*)(kt + b * 32 * 256 + k_addr[s]);
        f32x16 st[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
          for (int r = 0; r < 16; ++r) st[b][r] = 0.f;
#pragma unroll
          for (int s = 0; s < 8; ++s)
            st[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[b][s]), qf[s], st[b], 0, 0, 0);
        }
        if (kbase + 64 > a.n_g) {  // ragged: its first key exists, the rest may not
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (kbase + 32 * b + 8 * (r >> 2) + 4 * g + (r & 3) >= a.n_g) st[b][r] = -INFINITY;
        }
        float mx = st[0][0];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[b][r]);
        mx = max_halves(mx);
        const float mc = mx * c2;  // finite: key kbase exists
        float psum = 0.f;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) psum += __builtin_amdgcn_exp2f(fmaf(st[b][r], c2, -mc));
        psum = sum_halves(psum);
        const float m_new = fmaxf(m_run, mc);
        l_run = l_run * __builtin_amdgcn_exp2f(m_run - m_new) + psum * __builtin_amdgcn_exp2f(mc - m_new);
        m_run = m_new;
      }
      if (g == 0) partial[((size_t)h * n_kc + kc) * n_rows_pad + row] = make_float2(m_run, l_run);
    } else {
      // register r of the product holds row 8*(r/4) + 4*g + r%4 of the block for this lane's key
      float4 ls[4];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) ls[q4] = *(const float4*)&lse_w[8 * q4 + 4 * g];
#pragma unroll
      for (int kb = 0; kb < WIN_MAX_KB; ++kb) {
        if (kb < n_kb) {
          const unsigned char* kt = smem + (size_t)kb * 32 * 256;
          bf16x8 kf[8];
#pragma unroll
          for (int s = 0; s < 8; ++s) kf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(kt + k_addr[s]));
          f32x16 sc;
#pragma unroll
          for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
          for (int s = 0; s < 8; ++s) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[s], kf[s], sc, 0, 0, 0);
          float acc = 0.f;
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            acc += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 0], c2, -ls[q4].x));
            acc += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 1], c2, -ls[q4].y));
            acc += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 2], c2, -ls[q4].z));
            acc += __builtin_amdgcn_exp2f(fmaf(sc[4 * q4 + 3], c2, -ls[q4].w));
          }
          colsum[kb] += acc;
        }
      }
    }
  }
  if (!staged) {  // a wavefront without row blocks still takes part in the barriers
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __syncthreads();
  }
  if (PASS == 1) return;
#pragma unroll
  for (int kb = 0; kb < WIN_MAX_KB; ++kb) {
    if (kb < n_kb) {
      const float c = sum_halves(colsum[kb]);
      if (g == 0) red[wave * kc_keys + kb * 32 + l32] = c;
    }
  }
  __syncthreads();
  if (tid < kc_keys && k0 + tid < a.n_g) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < WIN_NW; ++w) s += red[w * kc_keys + tid];
    a.scores[(size_t)h * a.n_g + k0 + tid] = s;
  }
}

bool window_mfma_supported(int dtype, int h_q, int h_kv, int d, int w) {
  const long long q_bytes = (long long)w * h_q * d * 2;  // 32-bit byte offsets into the window tensor
  return dtype == QP_BF16 && d == WIN_D && win_rows_padded(h_q, h_kv, w) <= WIN_MAX_ROWS && q_bytes < (1ll << 31);
}

size_t window_mfma_workspace_bytes(int h_q, int h_kv, int n_g, int w) {
  const size_t n_kc = (n_g + WIN_KC_MIN - 1) / WIN_KC_MIN;  // an upper bound of the chunk count for any n_g
  const size_t rows = win_rows_padded(h_q, h_kv, w);
  return (size_t)h_kv * n_kc * rows * sizeof(float2);
}

void launch_score_window_mfma(const WindowArgs& a, hipStream_t s) {
  const int kc_keys = win_chunk_keys(a.n_g);
  const int n_kc = (a.n_g + kc_keys - 1) / kc_keys;
  float2* partial = (float2*)a.workspace;
  int wgs = n_kc * a.h_kv;
  if (8 % a.h_kv == 0) {
    const int per = 8 / a.h_kv;
    wgs = (n_kc + per - 1) / per * 8;
  }
  const size_t lds1 = (size_t)kc_keys * 256;
  const size_t lds2 = lds1 + (size_t)WIN_NW * 32 * sizeof(float) + (size_t)WIN_NW * kc_keys * sizeof(float);
  static bool attr_set[QP_MAX_DEVICES] = {};
  const int dev = current_device();
  if (dev < 0 || !attr_set[dev]) {
    const int max2 = WIN_KC_MAX * 256 + WIN_NW * 32 * (int)sizeof(float) + WIN_NW * WIN_KC_MAX * (int)sizeof(float);
    (void)hipFuncSetAttribute((const void*)window_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, WIN_KC_MAX * 256);
    (void)hipFuncSetAttribute((const void*)window_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, max2);
    if (dev >= 0) attr_set[dev] = true;
  }
  hipLaunchKernelGGL(window_kernel<1>, dim3(wgs), dim3(WIN_NT), lds1, s, a, partial, kc_keys, n_kc);
  hipLaunchKernelGGL(window_kernel<2>, dim3(wgs), dim3(WIN_NT), lds2, s, a, partial, kc_keys, n_kc);
}

}  // namespace qp
