// Decode-shaped group attention on bf16 MFMA (head_dim 128): at most 32 stacked rows per KV head, i.e. a
// "group" of one or a few new tokens attending to the whole pruned cache plus itself (Sec. 2.1 of the paper:
// the decoding stage that consumes the cache QuickPrefill builds). Same mathematics as attend_mfma_kernel.
//
// The cache's K and V are read exactly once and nothing is reused, so the kernel is shaped for HBM, not for the
// matrix pipe: no workgroup-shared tiles and no barrier in the loop. Keys are cut into blocks of 32; a workgroup
// takes a run of blocks and deals them to its 4 wavefronts, each of which works alone on its own 32 KB of LDS:
//   K, V block  global -> LDS with direct loads (XOR-swizzled 16-byte chunks, as in the large kernel), two buffers
//               each, refilled half by half: K two blocks ahead as soon as the QK product has its fragments, V two
//               blocks ahead after the PV product. All loads of the loop are
//               issued from inline assembly and waited for by count (the compiler tracks none of them, so it
//               neither drains the prefetch before an LDS read nor touches a register whose load is in flight);
//   S^T = K . Q^T with v_mfma_f32_32x32x16_bf16 (the <= 32 rows are the columns), online softmax per wavefront as
//   in the large kernel (a lane holds one row), V^T read back with ds_read_tr16_b64 for O^T += V^T . P^T.
// At the end the wavefronts' partial (max, sum, O) meet in LDS; the workgroup either writes the rows' final output
// (one workgroup per KV head) or a normalised partial + log2-sum-exp per chunk, merged by attend_merge_kernel like
// the key split of the large kernel. The group's own keys (causal among themselves) form the last block.
//
// F8 (the pruned cache in 8-bit E4M3): a cache block cannot go global -> LDS directly. The wavefront loads it into
// registers one block ahead with ordinary loads (8 bytes per lane, key and tensor: half the bytes of a bf16 block),
// widens it exactly to bf16 and writes it to its own LDS buffer in the same swizzled layout, so that the products
// and the softmax are the same code; the group's own block is bf16 and still loaded directly. The call is bound by
// the cache's bytes, which this halves.
#include "qp_internal.h"

#include <algorithm>

namespace qp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int DC_D = 128;
constexpr int DC_BK = 32;                  // keys per block
constexpr int DC_NW = 4;                   // wavefronts per workgroup
constexpr int DC_TILE = DC_BK * DC_D * 2;  // bytes of one K or V block in LDS
constexpr int DC_BUF = 2 * DC_TILE;        // K block + V block
constexpr int DC_WAVE_LDS = 2 * DC_BUF;    // two buffers per wavefront; the first 16 KB are reused for the final merge
constexpr int DC_MAX_ROWS = 32;
constexpr float DC_RESCALE_LOG2 = 8.f;

// s_waitcnt vmcnt(N) as a compiler-level memory barrier too: LDS reads of a block must not be hoisted above the
// wait for the direct loads that fill it.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// QK^T and online softmax of one 32-key block for this wavefront's rows (a lane holds row lane % 32 and half of the
// block's keys); leaves P^T (bf16) in pf. is_group: the block is the group's own keys (causal); n_valid: keys that
// exist in the block. The caller has waited for the block's K.
__device__ __forceinline__ void decode_qk_softmax(const unsigned char* kt, const int (&k_addr)[8], const bf16x8 (&qf)[8],
                                                  bool is_group, int n_valid, int t_lane, int g, float c2, float lazy,
                                                  float& m_run, float& l_run, f32x16 (&o)[4], bf16x8 (&pf)[2]) {
  u32x4 kf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) kf[s] = *(const u32x4*)(kt + k_addr[s]);
  f32x16 st;
#pragma unroll
  for (int r = 0; r < 16; ++r) st[r] = 0.f;
#pragma unroll
  for (int s = 0; s < 8; ++s)
    st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[s]), qf[s], st, 0, 0, 0);
  if (is_group || n_valid < DC_BK) {
    const int lim = is_group ? min(t_lane, n_valid - 1) : n_valid - 1;  // key_local <= lim is visible
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (8 * (r >> 2) + 4 * g + (r & 3) > lim) st[r] = -INFINITY;
  }
  float mx = st[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = fmaxf(mx, st[r]);
  mx = max_halves(mx);  // finite: key 0 of every block is visible to every row
  const float m_new = (mx > m_run + lazy) ? mx : m_run;
  const float mc = m_new * c2;
  bf16x2 ones;
  ones[0] = (__bf16)1.0f;
  ones[1] = (__bf16)1.0f;
  float psum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; r += 2) {
    bf16x2 pr;
    pr[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(st[r], c2, -mc));
    pr[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(st[r + 1], c2, -mc));
    psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
    pf[r >> 3][r & 7] = pr[0];
    pf[r >> 3][(r & 7) + 1] = pr[1];
  }
  if (__any(m_new != m_run)) {
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

// O^T += V^T . P^T for the block whose V sits at vt. The caller has waited for the block's V.
__device__ __forceinline__ void decode_pv(const unsigned char* vt, const int (&v_addr)[4], const bf16x8 (&pf)[2],
                                          f32x16 (&o)[4]) {
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      const unsigned char* p0 = vt + ks * 16 * 256 + v_addr[n];
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0 + 8 * 256));
      const s16x8 cat = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      o[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cat), pf[ks], o[n], 0, 0, 0);
    }
}

template <bool F8>
__global__ __launch_bounds__(DC_NW * 64) void attend_decode_kernel(AttendArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ float sm_m[DC_NW][DC_MAX_ROWS], sm_l[DC_NW][DC_MAX_ROWS];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform for the compiler too: block choice, pointers
  const int l32 = lane & 31, g = lane >> 5;
  const int h = blockIdx.y, chunk = blockIdx.x;
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = a.n_g * r_heads;  // <= 32, checked by the launcher
  const bool row_ok = l32 < n_rows;
  const int rowc = row_ok ? l32 : n_rows - 1;
  const int t_lane = rowc / r_heads, j_lane = rowc - t_lane * r_heads;
  const bf16_t* qrow = (const bf16_t*)a.q + ((size_t)t_lane * a.h_q + (size_t)h * r_heads + j_lane) * DC_D;
  bf16x8 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) qf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + 16 * s + 8 * g));

  constexpr int CROW = F8 ? DC_D : DC_D * 2;  // bytes of one cached row
  const unsigned char* ck = (const unsigned char*)a.ck + (size_t)h * a.cap * CROW;
  const unsigned char* cv = (const unsigned char*)a.cv + (size_t)h * a.cap * CROW;
  const unsigned char* gk = (const unsigned char*)a.k + (size_t)h * (DC_D * 2);
  const unsigned char* gv = (const unsigned char*)a.v + (size_t)h * (DC_D * 2);
  const unsigned gstride_b = (unsigned)a.h_kv * (DC_D * 2);
  const int n_cb = (a.c + DC_BK - 1) / DC_BK;  // cache blocks; block n_cb is the group's own keys
  const int b_end = min(n_cb + 1, (chunk + 1) * a.split_tiles);
  unsigned char* vbuf = smem + wave * DC_WAVE_LDS;

  // staging: load i of a block moves keys 4i .. 4i+3; this lane fills LDS position (lane & 15) of key 4i + (lane >> 4)
  // with the chunk that the swizzle puts there
  const int st_sub = lane >> 4, st_pos = lane & 15;
  // K fragment of d-step s: key l32, chunk 2s+g at position (2s+g) ^ (l32 & 15)
  int k_addr[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) k_addr[s] = l32 * 256 + (((2 * s + g) ^ (l32 & 15)) << 4);
  // V^T fragment addresses inside a block (same layout as the large kernel's tiles)
  const int l16 = lane & 15, grp = lane >> 4;
  const int v_key = 4 * (grp >> 1) + (l16 >> 2);
  int v_addr[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
    v_addr[n] = v_key * 256 + (((4 * n + 2 * (grp & 1) + ((l16 & 3) >> 1)) ^ ((v_key & 7) << 1)) << 4) + (l16 & 1) * 8;

  f32x16 o[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[n][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c2 = a.scale_log2;
  const float lazy = DC_RESCALE_LOG2 / c2;

  // request the K (V) half of block b_ into buffer buf_: 8 direct loads, each moving 4 keys x 256 bytes
#define QP_DC_REQUEST(b_, buf_, is_v_)                                                                   \
  {                                                                                                      \
    const bool grp_ = (b_) == n_cb;                                                                      \
    const int key0_ = grp_ ? 0 : (b_)*DC_BK;                                                             \
    const int last_ = grp_ ? a.n_g - 1 : a.c - 1; /* keys past the end are clamped: masked below */      \
    const unsigned stride_ = grp_ ? gstride_b : (unsigned)(DC_D * 2);                                    \
    const unsigned char* src_ = (is_v_) ? (grp_ ? gv : cv) : (grp_ ? gk : ck);                           \
    unsigned char* dst_ = vbuf + (buf_)*DC_BUF + ((is_v_) ? DC_TILE : 0);                                \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                      \
      const int kl_ = 4 * i + st_sub;                                                                    \
      const unsigned row_ = (unsigned)min(key0_ + kl_, last_) * stride_;                                 \
      const int swz_ = (is_v_) ? ((kl_ & 7) << 1) : (kl_ & 15);                                          \
      lds_dma16(src_, row_ + (unsigned)((st_pos ^ swz_) << 4), dst_ + i * 1024);                         \
    }                                                                                                    \
  }

  if constexpr (F8) {
    // 8-bit cache blocks through registers: 16 pieces of 8 bytes per lane and block (keys 4i + (lane >> 4), the
    // global chunk that belongs at LDS position lane & 15), requested one block ahead
    uint2 rk[8], rv[8];
    auto load_block = [&](int b_) {
      const int key0 = b_ * DC_BK, last = a.c - 1;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int kl = 4 * i + st_sub;
        const unsigned row = (unsigned)min(key0 + kl, last) * (unsigned)DC_D;  // keys past the end are clamped: masked below
        rk[i] = *(const uint2*)(ck + row + ((st_pos ^ (kl & 15)) << 3));
        rv[i] = *(const uint2*)(cv + row + ((st_pos ^ ((kl & 7) << 1)) << 3));
      }
    };
    auto widen8 = [](uint2 p) -> u32x4 {  // 8 E4M3 bytes -> 8 bf16 (the f32 values are exact; their high halves are the bf16)
      const auto a0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)p.x, false), a1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)p.x, true);
      const auto b0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)p.y, false), b1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)p.y, true);
      u32x4 o4;
      o4.x = (__float_as_uint(a0[0]) >> 16) | (__float_as_uint(a0[1]) & 0xffff0000u);
      o4.y = (__float_as_uint(a1[0]) >> 16) | (__float_as_uint(a1[1]) & 0xffff0000u);
      o4.z = (__float_as_uint(b0[0]) >> 16) | (__float_as_uint(b0[1]) & 0xffff0000u);
      o4.w = (__float_as_uint(b1[0]) >> 16) | (__float_as_uint(b1[1]) & 0xffff0000u);
      return o4;
    };
    int b = chunk * a.split_tiles + wave;
    int cur = 0;
    if (b < b_end && b < n_cb) load_block(b);
    while (b < b_end) {
      unsigned char* buf = vbuf + cur * DC_BUF;
      const bool has1 = b + DC_NW < b_end;
      if (b < n_cb) {
        // this block's pieces have arrived (requested a block ago): widen them into the buffer, then request the next
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          *(u32x4*)(buf + i * 1024 + lane * 16) = widen8(rk[i]);
          *(u32x4*)(buf + DC_TILE + i * 1024 + lane * 16) = widen8(rv[i]);
        }
        if (has1 && b + DC_NW < n_cb) load_block(b + DC_NW);
      } else {
        QP_DC_REQUEST(b, cur, false)  // the group's own keys and values: bf16, loaded directly
        QP_DC_REQUEST(b, cur, true)
        wait_vmcnt<0>();
      }
      bf16x8 pf[2];
      decode_qk_softmax(buf, k_addr, qf, b == n_cb, b == n_cb ? a.n_g : min(DC_BK, a.c - b * DC_BK), t_lane, g, c2, lazy,
                        m_run, l_run, o, pf);
      decode_pv(buf + DC_TILE, v_addr, pf, o);
      b += DC_NW;
      cur ^= 1;
    }
  } else {
    // The Q fragments (ordinary loads) must have arrived before the first request: from here on only untracked
    // operations are in flight, and the counts in the waits are exact.
    wait_vmcnt<0>();
    // Each half of a buffer is refilled as soon as its block has been consumed: K(i+2) right after the QK product of
    // block i, V(i+2) after its PV product, so that up to three halves beyond the current block are in flight.
    // Requests in issue order: K(i) V(i) K(i+1) V(i+1) | K(i+2) after QK(i) | V(i+2) after PV(i) ...
    int b = chunk * a.split_tiles + wave;
    int cur = 0;
    if (b < b_end) {
      QP_DC_REQUEST(b, 0, false)
      QP_DC_REQUEST(b, 0, true)
      if (b + DC_NW < b_end) {
        QP_DC_REQUEST(b + DC_NW, 1, false)
        QP_DC_REQUEST(b + DC_NW, 1, true)
      }
    }
    while (b < b_end) {
      const bool has1 = b + DC_NW < b_end, has2 = b + 2 * DC_NW < b_end;
      unsigned char* buf = vbuf + cur * DC_BUF;
      // K(i) has landed: V(i) and block i+1 (16 requests) may still be in flight
      if (has1) wait_vmcnt<24>();
      else wait_vmcnt<8>();
      bf16x8 pf[2];
      decode_qk_softmax(buf, k_addr, qf, b == n_cb, b == n_cb ? a.n_g : min(DC_BK, a.c - b * DC_BK), t_lane, g, c2, lazy,
                        m_run, l_run, o, pf);
      if (has2) QP_DC_REQUEST(b + 2 * DC_NW, cur, false)  // the K fragments of block i are in registers
      // V(i) has landed: block i+1 and K(i+2) may still be in flight
      if (has2) wait_vmcnt<24>();
      else if (has1) wait_vmcnt<16>();
      else wait_vmcnt<0>();
      decode_pv(buf + DC_TILE, v_addr, pf, o);
      if (has2) QP_DC_REQUEST(b + 2 * DC_NW, cur, true)
      b += DC_NW;
      cur ^= 1;
    }
  }
#undef QP_DC_REQUEST

  // the wavefronts' partial results meet in LDS (the start of each wavefront's buffers becomes its 32 x 128 f32 slab)
  wait_vmcnt<0>();
  __syncthreads();
  const float l_tot = sum_halves(l_run);
  if (row_ok) {
    float* slab = (float*)vbuf + l32 * DC_D;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)  // registers 4 q4 .. 4 q4 + 3 hold d = 32 n + 8 q4 + 4 g + 0..3
        *(float4*)(slab + 32 * n + 8 * q4 + 4 * g) =
            make_float4(o[n][4 * q4], o[n][4 * q4 + 1], o[n][4 * q4 + 2], o[n][4 * q4 + 3]);
    if (g == 0) {
      sm_m[wave][l32] = m_run * c2;  // -inf for a wavefront that had no block: weight 0 below
      sm_l[wave][l32] = l_tot;
    }
  }
  __syncthreads();
  const int d = tid & (DC_D - 1);
  const size_t total = (size_t)a.h_kv * n_rows;
  for (int row = tid >> 7; row < n_rows; row += (DC_NW * 64) >> 7) {
    float mw[DC_NW], big = -INFINITY;
#pragma unroll
    for (int w = 0; w < DC_NW; ++w) {
      mw[w] = sm_m[w][row];
      big = fmaxf(big, mw[w]);
    }
    float den = 0.f, acc = 0.f;  // at least one wavefront had a block, so big is finite
#pragma unroll
    for (int w = 0; w < DC_NW; ++w) {
      const float wgt = __builtin_amdgcn_exp2f(mw[w] - big);
      den = fmaf(wgt, sm_l[w][row], den);
      acc = fmaf(wgt, ((const float*)(smem + w * DC_WAVE_LDS))[row * DC_D + d], acc);
    }
    const int t = row / r_heads, j = row - t * r_heads;
    if (a.n_split > 1) {
      const size_t prow = (size_t)chunk * total + (size_t)h * n_rows + row;
      a.part_o[prow * DC_D + d] = acc / den;
      if (d == 0) a.part_lse[prow] = big + log2f(den);
    } else {
      ((bf16_t*)a.out)[((size_t)t * a.h_q + (size_t)h * r_heads + j) * DC_D + d] = f32_to_bf16_rne(acc / den);
      if (a.lse != nullptr && d == 0)
        a.lse[(size_t)(h * r_heads + j) * a.n_g + t] = (big + log2f(den)) * 0.6931471805599453f;
    }
  }
}

bool attend_decode_applies(const AttendArgs& a, int dtype) {
  return attend_mfma_supported(a, dtype) && a.n_g * (a.h_q / a.h_kv) <= DC_MAX_ROWS;
}

// Blocks per workgroup and workgroups per KV head: about one workgroup per compute unit in total, at least one
// block per wavefront; a single workgroup per head writes the output itself and needs no scratch.
AttendPlan plan_attend_decode(const AttendArgs& a, size_t split_ws_bytes) {
  AttendPlan p;
  const int n_rows = a.n_g * (a.h_q / a.h_kv);
  const int nb = (a.c + DC_BK - 1) / DC_BK + 1;
  const int per_head = std::max(1, device_cu_count() / a.h_kv);
  int bpw = std::max(DC_NW, (nb + per_head - 1) / per_head);
  int chunks = (nb + bpw - 1) / bpw;
  const size_t per_chunk = (size_t)a.h_kv * n_rows * (DC_D + 1) * sizeof(float);
  if (chunks > 1 && (size_t)chunks * per_chunk > split_ws_bytes) {  // not enough scratch: fewer, longer chunks
    const int fit = (int)std::min<size_t>(split_ws_bytes / per_chunk, (size_t)chunks);
    chunks = fit >= 2 ? fit : 1;
    bpw = (nb + chunks - 1) / chunks;
    chunks = (nb + bpw - 1) / bpw;
  }
  p.workgroups = chunks;
  p.n_split = chunks;
  p.split_rb = 0;
  p.split_tiles = bpw;
  p.mirrored = 0;
  p.scratch_bytes = chunks > 1 ? (size_t)chunks * per_chunk : 0;
  return p;
}

void launch_attend_decode(const AttendArgs& a_in, void* split_ws, size_t split_ws_bytes, hipStream_t s) {
  static bool attr_set[QP_MAX_DEVICES] = {};
  const int dev = current_device();
  if (dev < 0 || !attr_set[dev]) {
    (void)hipFuncSetAttribute((const void*)attend_decode_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              DC_NW * DC_WAVE_LDS);
    (void)hipFuncSetAttribute((const void*)attend_decode_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              DC_NW * DC_WAVE_LDS);
    if (dev >= 0) attr_set[dev] = true;
  }
  AttendArgs a = a_in;
  const AttendPlan p = plan_attend_decode(a, split_ws != nullptr ? split_ws_bytes : 0);
  a.n_split = p.n_split;
  a.split_tiles = p.split_tiles;
  a.split_rb = 0;
  a.part_rows = a.n_g * (a.h_q / a.h_kv);  // the merge covers every row
  a.mirrored = 0;
  a.part_o = nullptr;
  a.part_lse = nullptr;
  if (p.n_split > 1) {
    const size_t rows_total = (size_t)a.h_kv * a.n_g * (a.h_q / a.h_kv);
    a.part_o = (float*)split_ws;
    a.part_lse = a.part_o + (size_t)p.n_split * rows_total * DC_D;
  }
  if (a.cache_fp8)
    hipLaunchKernelGGL(attend_decode_kernel<true>, dim3(p.n_split, a.h_kv), dim3(DC_NW * 64), DC_NW * DC_WAVE_LDS, s, a);
  else
    hipLaunchKernelGGL(attend_decode_kernel<false>, dim3(p.n_split, a.h_kv), dim3(DC_NW * 64), DC_NW * DC_WAVE_LDS, s, a);
  if (p.n_split > 1) launch_attend_merge(a, s);
}

}  // namespace qp
