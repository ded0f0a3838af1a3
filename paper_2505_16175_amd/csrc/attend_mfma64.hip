// bf16 MFMA group attention, 64 rows per wavefront (gfx950, head_dim 128).
//
// Same mathematics, row stacking, key segments, swizzled direct-to-LDS tiles and fragment
// layouts as attend_mfma_v3_kernel (see attend_mfma.hip); what changes is the shape of the work
// a wavefront owns, chosen from measurements of that kernel:
//   * LDS bandwidth was the co-critical resource: with 32 rows per wavefront every 16-byte K or V
//     fragment read from LDS feeds one MFMA, and 8 wavefronts x 32 KB per 64-key tile keep the
//     128 B/clk LDS as busy as the matrix pipe. Here a wavefront owns TWO 32-row blocks, so each
//     fragment feeds two MFMAs and LDS traffic per flop halves.
//   * That needs ~400 registers, i.e. one wavefront per SIMD (4 per workgroup, 256 rows). The
//     overlap of matrix and vector work that two resident wavefronts never delivered is built into
//     the instruction stream instead: the two row blocks leapfrog,
//         QK(block 0) | QK(block 1) + softmax(block 0) | PV(block 0) + softmax(block 1) | PV(block 1)
//     so vector instructions sit between independent MFMAs of the other block.
#include "qp_internal.h"

namespace qp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int W_D = 128;                   // head_dim
constexpr int W_BN = 64;                   // keys per tile
constexpr int W_NW = 4;                    // wavefronts per workgroup
constexpr int W_NT = W_NW * 64;
constexpr int W_BM = W_NW * 64;            // rows per workgroup
constexpr int W_TILE = W_BN * 256;         // bytes of one K or V tile (unpadded, swizzled)
constexpr int W_LDS = 2 * 2 * W_TILE;      // K and V, double-buffered
constexpr float W_RESCALE_LOG2 = 8.f;      // move the reference max only when it grows by more than 2^8

// Softmax of one 32-row block of a tile. st: S^T (two 32-key blocks). Leaves P^T in pf, updates the
// block's running reference max / denominator share and rescales its O^T when the reference moved.
__device__ __forceinline__ void softmax_block(f32x16 (&st)[2], bool need_mask, int lim_local, int g, float c2,
                                              float lazy, bf16x2 ones, float& m_run, float& l_run, f32x16 (&o)[4],
                                              bf16x8 (&pf)[4]) {
  if (need_mask) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (kb * 32 + 8 * (r >> 2) + 4 * g + (r & 3) > lim_local) st[kb][r] = -INFINITY;
  }
  float mx = st[0][0];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[kb][r]);
  {
    // the other half of this row's keys lives in lane ^ 32
    const unsigned u = __builtin_bit_cast(unsigned, mx);
    const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    mx = fmaxf(__builtin_bit_cast(float, sw[0]), __builtin_bit_cast(float, sw[1]));
  }
  // first tile: m_run = -inf, so the max is adopted; key 0 is visible to every row, so it is finite
  const float m_new = (mx > m_run + lazy) ? mx : m_run;
  const float mc = m_new * c2;
  float psum = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      bf16x2 pr;
      pr[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(st[kb][r], c2, -mc));
      pr[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(st[kb][r + 1], c2, -mc));
      psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
      pf[kb * 2 + (r >> 3)][r & 7] = pr[0];
      pf[kb * 2 + (r >> 3)][(r & 7) + 1] = pr[1];
    }
  if (__builtin_expect(__any(m_new != m_run), 0)) {  // rare: a few times per row
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
    l_run *= alpha;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[n][r] *= alpha;
    m_run = m_new;
  }
  l_run += psum;
}

__global__ __launch_bounds__(W_NT, 1) void attend_mfma64_kernel(AttendArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int r_heads = a.h_q / a.h_kv;
  const int h = blockIdx.y;
  const int n_rows = a.n_g * r_heads;
  const int n_rb = (n_rows + W_BM - 1) / W_BM;
  const int rb = n_rb - 1 - (int)blockIdx.x;  // heaviest (latest tokens) first
  const int row0_wg = rb * W_BM;
  const int row0 = row0_wg + wave * 64;

  // this lane's two rows (one per 32-row block)
  int t_lane[2], j_lane[2];
  bool row_ok[2];
  bf16x8 qf[2][8];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int row = row0 + 32 * b + l32;
    row_ok[b] = row < n_rows;
    const int rowc = row_ok[b] ? row : n_rows - 1;
    t_lane[b] = rowc / r_heads;
    j_lane[b] = rowc - t_lane[b] * r_heads;
    const bf16_t* qrow = (const bf16_t*)a.q + ((size_t)t_lane[b] * a.h_q + (size_t)h * r_heads + j_lane[b]) * W_D;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[b][s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + 16 * s + 8 * g));
  }
  // wave-uniform token horizons
  const int t_w_max = min(row0 + 63, n_rows - 1) / r_heads;
  const int t_w_min = min(row0, n_rows - 1) / r_heads;
  const int t_wg_max = min(row0_wg + W_BM - 1, n_rows - 1) / r_heads;
  const bool wave_live = row0 < n_rows;
  const int n_ct = (a.c + W_BN - 1) / W_BN;        // cache tiles
  const int n_tiles = n_ct + t_wg_max / W_BN + 1;  // + group tiles

  const unsigned char* ck = (const unsigned char*)a.ck + (size_t)h * a.cap * (W_D * 2);
  const unsigned char* cv = (const unsigned char*)a.cv + (size_t)h * a.cap * (W_D * 2);
  const unsigned char* gk = (const unsigned char*)a.k + (size_t)h * (W_D * 2);
  const unsigned char* gv = (const unsigned char*)a.v + (size_t)h * (W_D * 2);
  const unsigned gstride_b = (unsigned)a.h_kv * (W_D * 2);

  // staging: this wavefront's four load instructions per tensor cover keys 16*wave .. 16*wave+15 of the tile;
  // instruction i: keys 16*wave + 4 i + (lane >> 4), LDS position lane & 15 <- global chunk position ^ swizzle(key)
  const int st_key = 16 * wave + (lane >> 4);
  const int st_pos = lane & 15;
  unsigned st_kc[4], st_vc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int key = st_key + 4 * i;
    st_kc[i] = (unsigned)((st_pos ^ (key & 15)) * 16);
    st_vc[i] = (unsigned)((st_pos ^ ((key & 7) << 1)) * 16);
  }

#define QP_W_ISSUE(tile_, buf_)                                                                                \
  {                                                                                                            \
    const bool in_cache_ = (tile_) < n_ct;                                                                     \
    const int base_ = in_cache_ ? (tile_)*W_BN : ((tile_)-n_ct) * W_BN;                                        \
    const int last_ = in_cache_ ? a.c - 1 : a.n_g - 1; /* rows past the end are clamped: masked, never used */ \
    const unsigned stride_ = in_cache_ ? (unsigned)(W_D * 2) : gstride_b;                                      \
    const unsigned char* ksrc_ = in_cache_ ? ck : gk;                                                          \
    const unsigned char* vsrc_ = in_cache_ ? cv : gv;                                                          \
    unsigned char* kdst_ = smem + (buf_) * (2 * W_TILE) + wave * 4096;                                         \
    _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                                                         \
      const unsigned r_ = __umul24((unsigned)min(base_ + st_key + 4 * i_, last_), stride_);                    \
      __builtin_amdgcn_global_load_lds((glb_void*)(ksrc_ + (r_ + st_kc[i_])), (lds_void*)(kdst_ + i_ * 1024), 16, 0, 0); \
      __builtin_amdgcn_global_load_lds((glb_void*)(vsrc_ + (r_ + st_vc[i_])), (lds_void*)(kdst_ + W_TILE + i_ * 1024), 16, 0, 0); \
    }                                                                                                          \
  }

  // fragment read addresses (bytes inside a tile)
  int k_addr[8];  // K fragment of d-step s: key l32 (+32 per block), chunk 2s+g at position (2s+g) ^ (l32 & 15)
#pragma unroll
  for (int s = 0; s < 8; ++s) k_addr[s] = l32 * 256 + (((2 * s + g) ^ (l32 & 15)) << 4);
  const int l16 = lane & 15, grp = lane >> 4;
  const int v_key = 4 * (grp >> 1) + (l16 >> 2);  // key inside a 16-key step (second read: + 8)
  int v_addr[4];  // V^T fragment of d-block n: chunk 4n + 2(grp&1) + ((l16&3)>>1), half (l16&1)
#pragma unroll
  for (int n = 0; n < 4; ++n)
    v_addr[n] = v_key * 256 + (((4 * n + 2 * (grp & 1) + ((l16 & 3) >> 1)) ^ ((v_key & 7) << 1)) << 4) + (l16 & 1) * 8;

  f32x16 o[2][4];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[b][n][r] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY};
  float l_run[2] = {0.f, 0.f};
  const float c2 = a.scale_log2;
  const float lazy = W_RESCALE_LOG2 / c2;
  bf16x2 ones;
  ones[0] = (__bf16)1.0f;
  ones[1] = (__bf16)1.0f;

  QP_W_ISSUE(0, 0)
  __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
  __syncthreads();

  for (int tile = 0; tile < n_tiles; ++tile) {
    const int buf = tile & 1;
    if (tile + 1 < n_tiles) QP_W_ISSUE(tile + 1, buf ^ 1)
    const bool in_cache = tile < n_ct;
    const int gt0 = (tile - n_ct) * W_BN;  // first group token of a group tile
    const bool live = wave_live && (in_cache || gt0 <= t_w_max);
    if (live) {
      const int cache_lim = a.c - 1 - tile * W_BN;
      const int lim0 = in_cache ? cache_lim : t_lane[0] - gt0;
      const int lim1 = in_cache ? cache_lim : t_lane[1] - gt0;
      const bool need_mask = in_cache ? (cache_lim < W_BN - 1) : (gt0 + W_BN - 1 > t_w_min);
      const unsigned char* kt = smem + buf * (2 * W_TILE);
      const unsigned char* vt = kt + W_TILE;

      // ---- K fragments (shared by both row blocks), then QK of block 0
      u32x4 kf[2][8];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s = 0; s < 8; ++s) kf[kb][s] = *(const u32x4*)(kt + kb * 32 * 256 + k_addr[s]);
      __builtin_amdgcn_sched_barrier(0);
      f32x16 st0[2], st1[2];
      const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
          st0[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[kb][s]), qf[0][s],
                                                            s == 0 ? zero16 : st0[kb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);

      // ---- QK of block 1 with the softmax of block 0 between its MFMAs
      bf16x8 pf0[4], pf1[4];
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
          st1[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[kb][s]), qf[1][s],
                                                            s == 0 ? zero16 : st1[kb], 0, 0, 0);
      softmax_block(st0, need_mask, lim0, g, c2, lazy, ones, m_run[0], l_run[0], o[0], pf0);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
        __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);  // 6 VALU
        __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);  // 2 transcendental
      }
      __builtin_amdgcn_sched_barrier(0);

      // ---- V^T fragments (shared by both row blocks), PV of block 0 with the softmax of block 1
      s16x8 vf[4][4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int n = 0; n < 4; ++n) {
          const unsigned char* p0 = vt + ks * 16 * 256 + v_addr[n];
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0 + 8 * 256));
          vf[ks][n] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int n = 0; n < 4; ++n)
          o[0][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[ks][n]), pf0[ks], o[0][n], 0, 0, 0);
      softmax_block(st1, need_mask, lim1, g, c2, lazy, ones, m_run[1], l_run[1], o[1], pf1);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // 2 LDS reads
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
        __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);  // 6 VALU
        __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);  // 2 transcendental
      }
      __builtin_amdgcn_sched_barrier(0);

      // ---- PV of block 1
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int n = 0; n < 4; ++n)
          o[1][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[ks][n]), pf1[ks], o[1][n], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wavefront's part of the next tile has landed in LDS
    __syncthreads();
  }
#undef QP_W_ISSUE

  if (!wave_live) return;
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const float l_tot = l_run[b] + __shfl_xor(l_run[b], 32, 64);
    if (row_ok[b]) {
      const float inv = 1.f / l_tot;
      bf16_t* orow = (bf16_t*)a.out + ((size_t)t_lane[b] * a.h_q + (size_t)h * r_heads + j_lane[b]) * W_D;
#pragma unroll
      for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          // registers 4*q4 .. 4*q4+3 hold d = 32 n + 8 q4 + 4 g + 0..3
          bf16x4 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(o[b][n][4 * q4 + e] * inv);
          *(uint2*)(orow + 32 * n + 8 * q4 + 4 * g) = __builtin_bit_cast(uint2, pk);
        }
      if (a.lse != nullptr && g == 0)
        a.lse[(size_t)(h * r_heads + j_lane[b]) * a.n_g + t_lane[b]] =
            (m_run[b] * c2 + log2f(l_tot)) * 0.6931471805599453f;
    }
  }
}

void launch_attend_mfma64(const AttendArgs& a, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)attend_mfma64_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS);
    attr_set = true;
  }
  const int n_rows = a.n_g * (a.h_q / a.h_kv);
  const int n_rb = (n_rows + W_BM - 1) / W_BM;
  hipLaunchKernelGGL(attend_mfma64_kernel, dim3(n_rb, a.h_kv), dim3(W_NT), W_LDS, s, a);
}

}  // namespace qp
