// bf16 MFMA group attention for gfx950 (head_dim 128), flash-style.
//
// What it computes (Sec. 3.2 of the paper, group-based prefill): for query head qh of KV head
// h = qh / R and group token t, softmax over {cache entries 0..C-1 of h} U {group tokens 0..t}
// of scale * q.k, times V.
//
// Mapping. The R query heads that share a KV head are stacked into one row space per KV head:
// row r = t * R + j (j = query head inside the KV group), which is also the memory order of
// Q_g[t][h*R + j][:]. A workgroup of NW wavefronts owns NW*32 consecutive rows of one KV head;
// every K/V tile it stages in LDS is therefore shared by all R query heads (GQA) and by NW*32/R
// tokens. Keys live in one index space kk: cache entries first (kk < C), then the group's own
// tokens (kk - C); row r sees kk <= C + t.
//
// Per wavefront (32 rows), per tile of 64 keys, with v_mfma_f32_32x32x16_bf16:
//   S^T[key][row] = K_tile . Q^T      (A = K from LDS, 16-byte reads; B = Q held in registers)
//     -> a lane holds ONE row (column of S^T) and 16 keys per 32-key block, so the softmax row
//        max / sum are in-register reductions plus one exchange between lane l and l+32.
//   P^T = exp2(c*S^T - c*m) rounded to bf16, fed straight back as the B operand of
//   O^T[d][row] += V^T . P^T         (A = V^T read from the row-major V tile in LDS with the
//                                      transposing ds_read_tr16_b64, 4 keys x 16 d per 16 lanes)
//     -> O^T keeps the lane <-> row association, so the online-softmax rescale is a per-lane
//        scalar multiply.
// The contraction index of the second product is permuted (keys 4g..4g+3 and 8+4g..8+4g+3 of
// each 16-key step go to lane half g) so that the accumulator layout of S^T is already the
// operand layout of P^T; V^T is read with the same permutation.
//
// K/V tiles are fetched global -> registers one tile ahead and written to a double-buffered LDS
// tile (one barrier per tile). Tiles beyond a wavefront's causal horizon are skipped by that
// wavefront; only tiles that straddle the diagonal (or the ragged end) are masked.
#include "qp_internal.h"

namespace qp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int MF_D = 128;      // head_dim
constexpr int MF_BN = 64;      // keys per tile
constexpr int MF_KS = 272;     // LDS row stride of the K tile in bytes (256 + 16: conflict-free 16-byte reads)
constexpr int MF_VS = 288;     // LDS row stride of the V tile in bytes (256 + 32: conflict-free transposing reads)
constexpr int MF_KBYTES = MF_BN * MF_KS;
constexpr int MF_VBYTES = MF_BN * MF_VS;

template <int NW>
__global__ __launch_bounds__(NW * 64) void attend_mfma_kernel(AttendArgs a) {
  constexpr int NT = NW * 64;
  constexpr int BM = NW * 32;
  constexpr int LOADS = (MF_BN * 16) / NT;  // 16-byte chunks of one tile per thread (per tensor)
  static_assert((MF_BN * 16) % NT == 0, "tile chunks must divide over the threads");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // [buf0: K | V][buf1: K | V]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int r_heads = a.h_q / a.h_kv;
  const int h = blockIdx.y;
  const int n_rows = a.n_g * r_heads;
  const int n_rb = (n_rows + BM - 1) / BM;
  const int rb = n_rb - 1 - (int)blockIdx.x;  // heaviest (latest tokens) first
  const int row0_wg = rb * BM;
  const int row0 = row0_wg + wave * 32;

  // this lane's row (column of S^T / O^T)
  const int row = row0 + l32;
  const bool row_ok = row < n_rows;
  const int rowc = row_ok ? row : n_rows - 1;
  const int t_lane = rowc / r_heads;
  const int j_lane = rowc - t_lane * r_heads;
  const int lim_lane = a.c + t_lane;  // visible keys: kk <= lim_lane
  const bf16_t* qrow = (const bf16_t*)a.q + ((size_t)t_lane * a.h_q + (size_t)h * r_heads + j_lane) * MF_D;

  // horizons (wave-uniform): tokens of the first and last row of the wave / workgroup
  const int last_row_w = min(row0 + 31, n_rows - 1);
  const int first_row_w = min(row0, n_rows - 1);
  const int lim_w_max = a.c + last_row_w / r_heads;
  const int lim_w_min = a.c + first_row_w / r_heads;
  const int last_row_wg = min(row0_wg + BM - 1, n_rows - 1);
  const int n_tiles = (a.c + last_row_wg / r_heads) / MF_BN + 1;
  const bool wave_live = row0 < n_rows;

  // Q^T operand: 8 k-steps of 16 d; this lane holds d = 16 s + 8 g .. + 7 of its row
  bf16x8 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    qf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + 16 * s + 8 * g));
  }

  const bf16_t* ck = (const bf16_t*)a.ck + (size_t)h * a.cap * MF_D;
  const bf16_t* cv = (const bf16_t*)a.cv + (size_t)h * a.cap * MF_D;
  const bf16_t* gk = (const bf16_t*)a.k + (size_t)h * MF_D;
  const bf16_t* gv = (const bf16_t*)a.v + (size_t)h * MF_D;
  const size_t gstride = (size_t)a.h_kv * MF_D;

  // Prefetch registers: named scalars of a native vector type (an array here ends up in scratch memory).
  static_assert(LOADS >= 1 && LOADS <= 4, "tile staging is written for 1..4 chunks per thread");
  u32x4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
// global -> registers, chunk i of tile `tile` (rows past the group's end are clamped: masked, never used)
#define QP_FETCH1(tile_, i_, kr_, vr_)                                                                      \
  if constexpr (LOADS > (i_)) {                                                                             \
    const int x = tid + NT * (i_);                                                                          \
    const int kk = (tile_)*MF_BN + (x >> 4);                                                                \
    const bool in_cache = kk < a.c;                                                                         \
    const size_t off =                                                                                      \
        (in_cache ? (size_t)kk * MF_D : (size_t)min(kk - a.c, a.n_g - 1) * gstride) + (size_t)((x & 15) * 8); \
    kr_ = *(const u32x4*)((in_cache ? ck : gk) + off);                                                      \
    vr_ = *(const u32x4*)((in_cache ? cv : gv) + off);                                                      \
  }
#define QP_FETCH(tile_)            \
  QP_FETCH1(tile_, 0, kr0, vr0)    \
  QP_FETCH1(tile_, 1, kr1, vr1)    \
  QP_FETCH1(tile_, 2, kr2, vr2)    \
  QP_FETCH1(tile_, 3, kr3, vr3)
// registers -> LDS buffer `buf`
#define QP_STAGE1(buf_, i_, kr_, vr_)                                                   \
  if constexpr (LOADS > (i_)) {                                                         \
    const int x = tid + NT * (i_);                                                      \
    unsigned char* kb = smem + (buf_) * (MF_KBYTES + MF_VBYTES);                        \
    *(u32x4*)(kb + (x >> 4) * MF_KS + (x & 15) * 16) = kr_;                             \
    *(u32x4*)(kb + MF_KBYTES + (x >> 4) * MF_VS + (x & 15) * 16) = vr_;                 \
  }
#define QP_STAGE(buf_)           \
  QP_STAGE1(buf_, 0, kr0, vr0)   \
  QP_STAGE1(buf_, 1, kr1, vr1)   \
  QP_STAGE1(buf_, 2, kr2, vr2)   \
  QP_STAGE1(buf_, 3, kr3, vr3)

  f32x16 o[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[n][r] = 0.f;
  float m_run = -INFINITY;  // running row max of the raw logits q.k (unscaled)
  float l_run = 0.f;        // this lane's share of the row's denominator
  const float c2 = a.scale_log2;

  // per-lane constant parts of the LDS read addresses
  const int k_off = l32 * MF_KS + g * 16;                                   // + kb*32*KS + s*32
  const int l16 = lane & 15, grp = lane >> 4;
  const int v_off = (4 * (grp >> 1) + (l16 >> 2)) * MF_VS + (16 * (grp & 1) + 4 * (l16 & 3)) * 2;  // + key0*VS + n*64

  QP_FETCH(0)
  QP_STAGE(0)
  __syncthreads();

  for (int tile = 0; tile < n_tiles; ++tile) {
    const int buf = tile & 1;
    if (tile + 1 < n_tiles) {
      QP_FETCH(tile + 1)
    }
    const int kk0 = tile * MF_BN;
    if (wave_live && kk0 <= lim_w_max) {
      const unsigned char* kb_base = smem + buf * (MF_KBYTES + MF_VBYTES);
      const unsigned char* vb_base = kb_base + MF_KBYTES;
      // ---- S^T = K . Q^T : two 32-key blocks
      f32x16 st[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) st[kb][r] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const u32x4 raw = *(const u32x4*)(kb_base + kb * 32 * MF_KS + k_off + s * 32);
          st[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), qf[s], st[kb], 0, 0, 0);
        }
      }
      // ---- mask (only tiles that reach past the earliest row's horizon)
      if (kk0 + MF_BN - 1 > lim_w_min) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kk = kk0 + kb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
            if (kk > lim_lane) st[kb][r] = -INFINITY;
          }
      }
      // ---- online softmax (this lane: one row, 32 of the tile's 64 keys; lane^32 has the others)
      float mx = st[0][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[kb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx);        // finite from tile 0 on: key 0 is visible to every row
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
      const float mc = m_new * c2;
      float psum = 0.f;
      bf16x8 pf[4];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(st[kb][r], c2, -mc));
          psum += p;
          pf[kb * 2 + (r >> 3)][r & 7] = (__bf16)p;
        }
      l_run = l_run * alpha + psum;
      if (__any(m_new != m_run)) {
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[n][r] *= alpha;
      }
      m_run = m_new;
      // ---- O^T += V^T . P^T : 4 key steps of 16 x 4 d-blocks of 32
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int n = 0; n < 4; ++n) {
          const unsigned char* p0 = vb_base + ks * 16 * MF_VS + v_off + n * 64;
          s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
          s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0 + 8 * MF_VS));
          const s16x8 cat = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cat), pf[ks], o[n], 0, 0, 0);
        }
      }
    }
    if (tile + 1 < n_tiles) {
      QP_STAGE(buf ^ 1)
    }
    __syncthreads();
  }

  if (!wave_live) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (!row_ok) return;
  const float inv = 1.f / l_tot;
  bf16_t* orow = (bf16_t*)a.out + ((size_t)t_lane * a.h_q + (size_t)h * r_heads + j_lane) * MF_D;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      // registers 4*q4 .. 4*q4+3 hold d = 32 n + 8 q4 + 4 g + 0..3
      bf16x4 pk;
#pragma unroll
      for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(o[n][4 * q4 + e] * inv);
      *(uint2*)(orow + 32 * n + 8 * q4 + 4 * g) = __builtin_bit_cast(uint2, pk);
    }
  if (a.lse != nullptr && g == 0)
    a.lse[(size_t)(h * r_heads + j_lane) * a.n_g + t_lane] = (m_run * c2 + log2f(l_tot)) * 0.6931471805599453f;
}

bool attend_mfma_supported(const AttendArgs& a, int dtype) {
  return dtype == QP_BF16 && a.d == MF_D && a.h_kv <= 65535;
}

void launch_attend_mfma(const AttendArgs& a, hipStream_t s) {
  constexpr int NW = 8;
  const int n_rows = a.n_g * (a.h_q / a.h_kv);
  const int n_rb = (n_rows + NW * 32 - 1) / (NW * 32);
  const size_t lds = 2 * (MF_KBYTES + MF_VBYTES);
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)attend_mfma_kernel<NW>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_set = true;
  }
  hipLaunchKernelGGL((attend_mfma_kernel<NW>), dim3(n_rb, a.h_kv), dim3(NW * 64), lds, s, a);
}

#undef QP_FETCH
#undef QP_FETCH1
#undef QP_STAGE1
#undef QP_STAGE

}  // namespace qp
