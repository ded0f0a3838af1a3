// bf16 MFMA matrix product for the projections of the decoder layer around the path (gfx950):
//   Y[m][n] = sum_k X[m][k] W[n][k]      X [M][K] activations (tokens slow), W [N][K] weights ([out][in]),
// f32 accumulation, with the layer's elementwise steps fused into the store:
//   PLAIN    Y (+ bias[n]) (+ residual[m][n]) -> bf16 [M][N]          (o_proj and down_proj with the residual add)
//   QKV_ROPE Y + bias, rotary embedding on the query and key heads, scattered to Q [M][H_q][128],
//            K [M][H_kv][128], V [M][H_kv][128] (the token-major layout the attention kernels read)
//   SWIGLU   W = [gate rows ; up rows] (2 d_ff rows): SiLU(gate) * up -> bf16 [M][d_ff]
//            (Appendix D.1 of the paper: SwiGLU(x) = W_down(SiLU(W_gate x) * W_up x))
//
// Tiling. A workgroup of 8 wavefronts owns a 256 x 256 output tile and walks K in steps of 64. Both operand
// tiles (256 rows x 128 bytes each) go global -> LDS with global_load_lds_dwordx4 into a ring of buffers, the
// next step's tiles in flight while this step's are multiplied; one barrier per step, placed before the step's last
// quarter of products so that the matrix pipe stays busy across it. Rows are unpadded; the
// 16-byte chunk c of row r sits at position c ^ ((r >> 1) & 7), which makes both the 1 KB stores of the loads
// and the fragment reads (32 rows x 16 bytes per half wavefront) conflict-free.
// Wavefront (wm, wn) of the 2 x 4 arrangement computes 128 tokens x 64 outputs as 4 x 2 blocks of
// v_mfma_f32_32x32x16_bf16 with the WEIGHT rows as the A operand and the token rows as B, so that a lane ends
// up with one token (m = lane & 31) and, per block, 16 outputs in runs of 4: stores are 8-byte runs of a token's
// row, and the fused steps below only ever combine values of the same lane:
//   * QKV_ROPE: the 256 tile columns are two heads; wavefront wn serves head wn >> 1 and, of its 128 dims, the
//     32 dims [32 (wn & 1), +32) in block 0 and their rotary partners (+64) in block 1. The weight rows are
//     fetched into LDS in that order (a permutation inside the tile, contiguous in runs of 32 rows).
//   * SWIGLU: block 0 holds gate columns [n0/2 + 32 wn, +32), block 1 the up columns of the same outputs.
// Workgroup ids are dealt round-robin over the 8 XCDs; the workgroups an XCD runs side by side cover a block of
// token tiles x weight tiles, which bounds what its L2 has to fetch per k-step.
#include <atomic>

#include "qp_internal.h"

namespace qp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#ifndef GM_BK
#define GM_BK 64
#endif
constexpr int GM_BN = 256;  // weight rows per tile
constexpr int GM_NW = 8;
// Token rows per tile BM: 256, or 128 for launches that would leave compute units idle with 256-row tiles.
// k per ring slot BK: 64 or 32. The ring is as deep as 160 KB of LDS allow; all its free slots are in flight.
template <int BM, int BK>
struct Tile {
  static constexpr int ROWB = BK * 2;                       // bytes per tile row
  static constexpr int CPR = ROWB / 16;                     // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;                      // rows one load instruction covers
  static constexpr int RPL = 256 / ROWB;                    // rows per 256 bytes of LDS (one sweep of the banks)
  static constexpr int KS = BK / 16;                        // k-steps of the MFMA per slot
  static constexpr int XT = BM * ROWB;                      // bytes of the activation tile
  static constexpr int STAGE = (BM + GM_BN) * ROWB;         // one ring slot: activation tile + weight tile
  static constexpr int STAGES = (160 * 1024) / STAGE < 6 ? (160 * 1024) / STAGE : 6;
  static constexpr int MI = BM / 64;                        // 32-token blocks per wavefront (wavefront rows: BM / 2)
  static constexpr int XQ = BM / 8 / RPI;                   // activation load instructions per wavefront and slot
  static constexpr int WQ = 32 / RPI;                       // weight load instructions per wavefront and slot
  static constexpr int PER_WAVE = XQ + WQ;
  // chunk c of row r sits at position c ^ swizzle(r): 16 consecutive rows' reads of one chunk index, and the 1 KB
  // written by one load instruction, then touch every bank group once
  __device__ static constexpr int swizzle(int r) { return (r / RPL) & (CPR - 1); }
};

// 64 lanes x 16 bytes global -> LDS at the wave-uniform LDS byte address lds_addr (lane L lands at lds_addr + 16 L);
// m0 is clobbered on purpose (see lds_dma16)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void gm_dma16(const unsigned char* base, unsigned byte_off, unsigned lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(byte_off), "s"(base), "s"(lds_addr)
      : "memory", "m0");
}
#pragma clang diagnostic pop

template <int N>
__device__ __forceinline__ void gm_wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// LDS row j of the weight tile <- which weight row (relative to the tile's first), per mode
template <int MODE>
__device__ __forceinline__ int weight_row(int j, int n0, int d_ff) {
  if (MODE == GEMM_QKV_ROPE) return n0 + (j & ~127) + ((j >> 5) & 1) * 64 + ((j >> 6) & 1) * 32 + (j & 31);
  if (MODE == GEMM_SWIGLU) return ((j >> 5) & 1) * d_ff + (n0 >> 1) + (j >> 6) * 32 + (j & 31);
  return n0 + j;
}

template <int MODE, int BM, int BK>
__global__ __launch_bounds__(GM_NW * 64) void gemm_bf16_kernel(GemmArgs a) {
  typedef Tile<BM, BK> T;
  constexpr int ROWB = T::ROWB;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g = lane >> 5;
  const int wm = wave >> 2, wn = wave & 3;

  // workgroup id -> (weight tile, token tile). Ids go round-robin over the 8 XCDs; the 32 workgroups that an XCD
  // runs side by side form a block of up to 8 token tiles x 4 weight tiles, so that per k-step the XCD's L2 fetches
  // 8 + 4 operand tiles for 32 products.
  const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
  const int mi = idx % a.m_block, t = idx / a.m_block;
  const int ni = t & 3, b = t >> 2;
  const int mc = b / a.n_quads, nq = b - mc * a.n_quads;
  const int tm = mc * a.m_block + mi, tn = xcd + 8 * (nq * 4 + ni);
  if (tm >= a.tiles_m || tn >= a.tiles_n) return;  // padding of the mapping (whole workgroup, before any barrier)
  const int m0 = tm * BM, n0 = tn * GM_BN;
  const int d_ff = a.n >> 1;

  // staging: activation load q of this wavefront covers tile rows (BM/8) wave + RPI q + lane / CPR, weight load q
  // rows 32 wave + RPI q + lane / CPR; LDS position lane % CPR of the row holds chunk position ^ swizzle(row)
  const unsigned char* xg = (const unsigned char*)a.x;
  const unsigned char* wg = (const unsigned char*)a.w;
  const size_t row_b = (size_t)a.k * 2;
  unsigned x_off[T::XQ], w_off[T::WQ];
  const int wb = MODE == GEMM_SWIGLU ? (n0 >> 1) : n0;  // first weight row this tile touches
  // offsets relative to the tile's first row (the launcher checks that they fit 32 bits)
#pragma unroll
  for (int q = 0; q < T::XQ; ++q) {
    const int r = (BM / 8) * wave + T::RPI * q + lane / T::CPR;
    const int xr = min(m0 + r, a.m - 1);  // rows past the end: computed, not stored
    x_off[q] = (unsigned)((size_t)(xr - m0) * row_b) + (unsigned)((lane % T::CPR) ^ T::swizzle(r)) * 16;
  }
#pragma unroll
  for (int q = 0; q < T::WQ; ++q) {
    const int r = 32 * wave + T::RPI * q + lane / T::CPR;
    const int wr = min(weight_row<MODE>(r, n0, d_ff), a.n - 1);
    w_off[q] = (unsigned)((size_t)(wr - wb) * row_b) + (unsigned)((lane % T::CPR) ^ T::swizzle(r)) * 16;
  }
  // contraction split (launches of few tiles): grid.y deals the k-steps to chunks, each leaving an f32 partial tile
  const int step_begin = blockIdx.y * a.steps_per_split;
  const unsigned char* x_base = xg + (size_t)m0 * row_b + (size_t)step_begin * ROWB;
  const unsigned char* w_base = wg + (size_t)wb * row_b + (size_t)step_begin * ROWB;
  const unsigned smem_lds = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const unsigned x_lds = smem_lds + wave * (BM / 8) * ROWB, w_lds = smem_lds + T::XT + wave * 32 * ROWB;

  // load instruction p_ of a step (activation loads first, then weight loads) into ring slot slot_
#define GM_ISSUE_ONE(p_, step_, slot_)                                                                          \
  {                                                                                                             \
    const unsigned koff_ = (unsigned)(step_) * ROWB;                                                         \
    if ((p_) < T::XQ) gm_dma16(x_base, x_off[(p_) < T::XQ ? (p_) : 0] + koff_, x_lds + (slot_)*T::STAGE + 1024 * (p_)); \
    else gm_dma16(w_base, w_off[(p_) - T::XQ] + koff_, w_lds + (slot_)*T::STAGE + 1024 * ((p_) - T::XQ));       \
  }
#define GM_ISSUE(step_, slot_) \
  { _Pragma("unroll") for (int p_ = 0; p_ < T::PER_WAVE; ++p_) GM_ISSUE_ONE(p_, step_, slot_) }

  // fragment addresses inside a slot: row (l32 + 32 block), chunk 2 s + g of k-step s
  int f_off[T::KS];
#pragma unroll
  for (int s = 0; s < T::KS; ++s) f_off[s] = l32 * ROWB + (((2 * s + g) ^ T::swizzle(l32)) << 4);
  const int x_frag = wm * (BM / 2) * ROWB;
  const int w_frag = T::XT + wn * 64 * ROWB;

  f32x16 acc[2][T::MI];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < T::MI; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  // Ring schedule. All slots are free at the start, so the first STAGES steps are requested at once. Inside the
  // loop the barrier sits before the LAST k-step's products of a step: by then every wavefront has read all its
  // fragments of the step (its slot can be refilled), the next step's tiles have landed, and the wait at the
  // barrier, the refill requests and the latency of the next step's first fragment reads all run under those
  // products instead of leaving the matrix pipe idle between steps.
  const int n_steps = min(a.steps_per_split, a.k / BK - step_begin);
  constexpr int S = T::STAGES, PW = T::PER_WAVE;
#pragma unroll
  for (int p = 0; p < S; ++p)
    if (p < n_steps) GM_ISSUE(p, p)
  // the first slot's tiles have landed: all but the min(S, n_steps) - 1 later requests are complete
  switch (n_steps < S ? n_steps : S) {
    case 1: gm_wait_vmcnt<0>(); break;
    case 2: gm_wait_vmcnt<PW>(); break;
    case 3: gm_wait_vmcnt<2 * PW>(); break;
    case 4: gm_wait_vmcnt<3 * PW>(); break;
    case 5: gm_wait_vmcnt<4 * PW>(); break;
    default: gm_wait_vmcnt<5 * PW>(); break;
  }
  __syncthreads();
  u32x4 wf[2][2], xf[2][T::MI];  // fragments of k-step s+1 are read while the products of k-step s run (two sets)
#define GM_READ(st_, s_, b_)                                                                                   \
  {                                                                                                            \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) wf[b_][j] = *(const u32x4*)((st_) + w_frag + j * 32 * ROWB + f_off[s_]); \
    _Pragma("unroll") for (int i = 0; i < T::MI; ++i) xf[b_][i] = *(const u32x4*)((st_) + x_frag + i * 32 * ROWB + f_off[s_]); \
  }
#define GM_MFMA(b_)                                                                                            \
  _Pragma("unroll") for (int i = 0; i < T::MI; ++i) _Pragma("unroll") for (int j = 0; j < 2; ++j) acc[j][i] =  \
      __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf[b_][j]), __builtin_bit_cast(bf16x8, xf[b_][i]), acc[j][i], 0, 0, 0);
  // one product / one fragment read, by index, so that the work after the barrier can be interleaved by hand
#define GM_MFMA_ONE(b_, mf_)                                                                                   \
  acc[(mf_) & 1][(mf_) >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                        \
      __builtin_bit_cast(bf16x8, wf[b_][(mf_) & 1]), __builtin_bit_cast(bf16x8, xf[b_][(mf_) >> 1]), acc[(mf_) & 1][(mf_) >> 1], 0, 0, 0);
#define GM_READ_ONE(st_, r_)                                                                                   \
  {                                                                                                            \
    if ((r_) < 2) wf[0][(r_) < 2 ? (r_) : 0] = *(const u32x4*)((st_) + w_frag + (r_) * 32 * ROWB + f_off[0]);   \
    else xf[0][(r_) >= 2 ? (r_) - 2 : 0] = *(const u32x4*)((st_) + x_frag + ((r_) - 2) * 32 * ROWB + f_off[0]); \
  }
  constexpr int NM = 2 * T::MI;                       // products per k-step
  constexpr int PIECES = PW + 2 + T::MI;              // refill requests + first fragment reads of the next step
  constexpr int PER = (PIECES + NM - 1) / NM;         // of them behind each product
  GM_READ(smem, 0, 0)
  int slot = 0;
  for (int step = 0; step + 1 < n_steps; ++step) {
    const unsigned char* st = smem + slot * T::STAGE;
#pragma unroll
    for (int s = 0; s < T::KS - 1; ++s) {
      GM_READ(st, s + 1, (s + 1) & 1)
      __builtin_amdgcn_sched_barrier(0);
      GM_MFMA(s & 1)
      __builtin_amdgcn_sched_barrier(0);
    }
    const int next = slot == S - 1 ? 0 : slot + 1;
    // this wavefront's part of the next step's tiles has landed (later steps' may still be in flight) ...
    {
      const int behind = n_steps - 2 - step < S - 2 ? n_steps - 2 - step : S - 2;  // requests that may stay in flight
      switch (behind) {
        case 0: gm_wait_vmcnt<0>(); break;
        case 1: gm_wait_vmcnt<PW>(); break;
        case 2: gm_wait_vmcnt<2 * PW>(); break;
        case 3: gm_wait_vmcnt<3 * PW>(); break;
        default: gm_wait_vmcnt<4 * PW>(); break;
      }
    }
    __syncthreads();  // ... everyone's has, and everyone has read its last fragments of this step's slot
    const bool refill = step + S < n_steps;
    const unsigned char* st_next = smem + next * T::STAGE;
#pragma unroll
    for (int mf = 0; mf < NM; ++mf) {
      GM_MFMA_ONE(1, mf)
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < PER; ++u) {
        const int p = mf * PER + u;
        if (p < PW) {
          if (refill) GM_ISSUE_ONE(p, step + S, slot)
        } else if (p < PIECES) {
          GM_READ_ONE(st_next, p - PW)
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    slot = next;
  }
  {  // last step: nothing left to request or to wait for
    const unsigned char* st = smem + slot * T::STAGE;
#pragma unroll
    for (int s = 0; s < T::KS - 1; ++s) {
      GM_READ(st, s + 1, (s + 1) & 1)
      __builtin_amdgcn_sched_barrier(0);
      GM_MFMA(s & 1)
      __builtin_amdgcn_sched_barrier(0);
    }
    GM_MFMA(1)
  }
#undef GM_MFMA_ONE
#undef GM_READ_ONE
#undef GM_ISSUE_ONE
#undef GM_READ
#undef GM_MFMA
#undef GM_ISSUE

  // ---- store: lane owns token m = m0 + (BM/2) wm + 32 i + l32 and, in block j, outputs 8 (r >> 2) + 4 g + (r & 3)
  if (a.split_k > 1) {
    // partial sums of this k chunk, f32 [chunk][m][n] with n the output's logical column (for QKV: head * 128 + dim);
    // gemm_reduce_kernel adds the chunks in order and applies the mode's store
    float* part = a.partial + (size_t)blockIdx.y * a.m * a.n;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        int n;
        if (MODE == GEMM_QKV_ROPE) n = ((n0 >> 7) + (wn >> 1)) * 128 + (wn & 1) * 32 + j * 64 + 8 * q4 + 4 * g;
        else n = n0 + wn * 64 + j * 32 + 8 * q4 + 4 * g;
        if (n >= a.n) continue;
#pragma unroll
        for (int i = 0; i < T::MI; ++i) {
          const int m = m0 + wm * (BM / 2) + i * 32 + l32;
          if (m >= a.m) continue;
          *(float4*)(part + (size_t)m * a.n + n) =
              make_float4(acc[j][i][4 * q4], acc[j][i][4 * q4 + 1], acc[j][i][4 * q4 + 2], acc[j][i][4 * q4 + 3]);
        }
      }
    return;
  }
  if (MODE == GEMM_PLAIN) {
    const bf16_t* bias = (const bf16_t*)a.bias;
    const bf16_t* res = (const bf16_t*)a.residual;
    bf16_t* out = (bf16_t*)a.out;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int n = n0 + wn * 64 + j * 32 + 8 * q4 + 4 * g;
        if (n >= a.n) continue;
        float b[4] = {0.f, 0.f, 0.f, 0.f};
        if (bias != nullptr) {
          const uint2 raw = *(const uint2*)(bias + n);
          b[0] = bf16lo_to_f32(raw.x), b[1] = bf16hi_to_f32(raw.x), b[2] = bf16lo_to_f32(raw.y), b[3] = bf16hi_to_f32(raw.y);
        }
#pragma unroll
        for (int i = 0; i < T::MI; ++i) {
          const int m = m0 + wm * (BM / 2) + i * 32 + l32;
          if (m >= a.m) continue;
          float y[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = acc[j][i][4 * q4 + e] + b[e];
          if (res != nullptr) {
            const uint2 raw = *(const uint2*)(res + (size_t)m * a.n + n);
            y[0] += bf16lo_to_f32(raw.x), y[1] += bf16hi_to_f32(raw.x), y[2] += bf16lo_to_f32(raw.y), y[3] += bf16hi_to_f32(raw.y);
          }
          bf16x4 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk[e] = (__bf16)y[e];
          *(uint2*)(out + (size_t)m * a.n + n) = __builtin_bit_cast(uint2, pk);
        }
      }
  } else if (MODE == GEMM_QKV_ROPE) {
    // head of this wavefront and where its rows go
    const int head = (n0 >> 7) + (wn >> 1);
    const int dim0 = (wn & 1) * 32;  // block 0: dims dim0 + ..., block 1: dim0 + 64 + ...
    const bf16_t* bias = (const bf16_t*)a.bias + (size_t)head * 128;
    bf16_t* dst;
    int heads_dst, head_dst;
    bool rotate = true;
    if (head < a.h_q) dst = (bf16_t*)a.q, heads_dst = a.h_q, head_dst = head;
    else if (head < a.h_q + a.h_kv) dst = (bf16_t*)a.k_out, heads_dst = a.h_kv, head_dst = head - a.h_q;
    else dst = (bf16_t*)a.v_out, heads_dst = a.h_kv, head_dst = head - a.h_q - a.h_kv, rotate = false;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int f = dim0 + 8 * q4 + 4 * g;  // rotary frequency index of the run's first element
      float b0[4], b1[4];
      {
        const uint2 r0 = *(const uint2*)(bias + f), r1 = *(const uint2*)(bias + 64 + f);
        b0[0] = bf16lo_to_f32(r0.x), b0[1] = bf16hi_to_f32(r0.x), b0[2] = bf16lo_to_f32(r0.y), b0[3] = bf16hi_to_f32(r0.y);
        b1[0] = bf16lo_to_f32(r1.x), b1[1] = bf16hi_to_f32(r1.x), b1[2] = bf16lo_to_f32(r1.y), b1[3] = bf16hi_to_f32(r1.y);
      }
#pragma unroll
      for (int i = 0; i < T::MI; ++i) {
        const int m = m0 + wm * (BM / 2) + i * 32 + l32;
        if (m >= a.m) continue;
        float lo[4], hi[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) lo[e] = acc[0][i][4 * q4 + e] + b0[e], hi[e] = acc[1][i][4 * q4 + e] + b1[e];
        if (rotate) {
          const float4 cs0 = *(const float4*)(a.cos_sin + ((size_t)m * 64 + f) * 2);
          const float4 cs1 = *(const float4*)(a.cos_sin + ((size_t)m * 64 + f + 2) * 2);
          const float c[4] = {cs0.x, cs0.z, cs1.x, cs1.z}, s[4] = {cs0.y, cs0.w, cs1.y, cs1.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float x0 = lo[e], x1 = hi[e];
            lo[e] = x0 * c[e] - x1 * s[e];
            hi[e] = x1 * c[e] + x0 * s[e];
          }
        }
        bf16x4 p0, p1;
#pragma unroll
        for (int e = 0; e < 4; ++e) p0[e] = (__bf16)lo[e], p1[e] = (__bf16)hi[e];
        bf16_t* row = dst + ((size_t)m * heads_dst + head_dst) * 128;
        *(uint2*)(row + f) = __builtin_bit_cast(uint2, p0);
        *(uint2*)(row + 64 + f) = __builtin_bit_cast(uint2, p1);
      }
    }
  } else {  // GEMM_SWIGLU
    bf16_t* out = (bf16_t*)a.out;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int n = (n0 >> 1) + wn * 32 + 8 * q4 + 4 * g;
#pragma unroll
      for (int i = 0; i < T::MI; ++i) {
        const int m = m0 + wm * (BM / 2) + i * 32 + l32;
        if (m >= a.m) continue;
        bf16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float gate = acc[0][i][4 * q4 + e], up = acc[1][i][4 * q4 + e];
          pk[e] = (__bf16)(gate / (1.f + __expf(-gate)) * up);
        }
        *(uint2*)(out + (size_t)m * d_ff + n) = __builtin_bit_cast(uint2, pk);
      }
    }
  }
}

// Second launch of a split contraction: sums the chunks' partial tiles in chunk order and applies the mode's store.
// One thread per token and run of 4 outputs (QKV_ROPE: per run of 4 dims of a head's first half and their rotary
// partners).
template <int MODE>
__global__ __launch_bounds__(256) void gemm_reduce_kernel(GemmArgs a) {
  const long id = (long)blockIdx.x * 256 + threadIdx.x;
  const int runs = MODE == GEMM_QKV_ROPE ? a.n / 8 : a.n / 4;  // per token
  if (id >= (long)a.m * runs) return;
  const int m = (int)(id / runs), r = (int)(id - (long)m * runs);
  const size_t stride = (size_t)a.m * a.n;
  if (MODE == GEMM_PLAIN) {
    const int n = 4 * r;
    const float* p = a.partial + (size_t)m * a.n + n;
    float4 y = *(const float4*)p;
    for (int c = 1; c < a.split_k; ++c) {
      const float4 t = *(const float4*)(p + c * stride);
      y.x += t.x, y.y += t.y, y.z += t.z, y.w += t.w;
    }
    if (a.bias != nullptr) {
      const uint2 raw = *(const uint2*)((const bf16_t*)a.bias + n);
      y.x += bf16lo_to_f32(raw.x), y.y += bf16hi_to_f32(raw.x), y.z += bf16lo_to_f32(raw.y), y.w += bf16hi_to_f32(raw.y);
    }
    if (a.residual != nullptr) {
      const uint2 raw = *(const uint2*)((const bf16_t*)a.residual + (size_t)m * a.n + n);
      y.x += bf16lo_to_f32(raw.x), y.y += bf16hi_to_f32(raw.x), y.z += bf16lo_to_f32(raw.y), y.w += bf16hi_to_f32(raw.y);
    }
    bf16x4 pk;
    pk[0] = (__bf16)y.x, pk[1] = (__bf16)y.y, pk[2] = (__bf16)y.z, pk[3] = (__bf16)y.w;
    *(uint2*)((bf16_t*)a.out + (size_t)m * a.n + n) = __builtin_bit_cast(uint2, pk);
  } else if (MODE == GEMM_QKV_ROPE) {
    const int head = r / 16, f = 4 * (r % 16);  // f: first of 4 rotary frequencies
    const float* p = a.partial + (size_t)m * a.n + head * 128 + f;
    float4 lo4 = *(const float4*)p, hi4 = *(const float4*)(p + 64);
    for (int c = 1; c < a.split_k; ++c) {
      const float4 t = *(const float4*)(p + c * stride), u = *(const float4*)(p + c * stride + 64);
      lo4.x += t.x, lo4.y += t.y, lo4.z += t.z, lo4.w += t.w;
      hi4.x += u.x, hi4.y += u.y, hi4.z += u.z, hi4.w += u.w;
    }
    float lo[4] = {lo4.x, lo4.y, lo4.z, lo4.w}, hi[4] = {hi4.x, hi4.y, hi4.z, hi4.w};
    const bf16_t* bias = (const bf16_t*)a.bias + (size_t)head * 128;
    const uint2 r0 = *(const uint2*)(bias + f), r1 = *(const uint2*)(bias + 64 + f);
    lo[0] += bf16lo_to_f32(r0.x), lo[1] += bf16hi_to_f32(r0.x), lo[2] += bf16lo_to_f32(r0.y), lo[3] += bf16hi_to_f32(r0.y);
    hi[0] += bf16lo_to_f32(r1.x), hi[1] += bf16hi_to_f32(r1.x), hi[2] += bf16lo_to_f32(r1.y), hi[3] += bf16hi_to_f32(r1.y);
    bf16_t* dst;
    int heads_dst, head_dst;
    if (head < a.h_q) dst = (bf16_t*)a.q, heads_dst = a.h_q, head_dst = head;
    else if (head < a.h_q + a.h_kv) dst = (bf16_t*)a.k_out, heads_dst = a.h_kv, head_dst = head - a.h_q;
    else dst = (bf16_t*)a.v_out, heads_dst = a.h_kv, head_dst = head - a.h_q - a.h_kv;
    if (head < a.h_q + a.h_kv) {
      const float4 cs0 = *(const float4*)(a.cos_sin + ((size_t)m * 64 + f) * 2);
      const float4 cs1 = *(const float4*)(a.cos_sin + ((size_t)m * 64 + f + 2) * 2);
      const float c[4] = {cs0.x, cs0.z, cs1.x, cs1.z}, sn[4] = {cs0.y, cs0.w, cs1.y, cs1.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float x0 = lo[e], x1 = hi[e];
        lo[e] = x0 * c[e] - x1 * sn[e];
        hi[e] = x1 * c[e] + x0 * sn[e];
      }
    }
    bf16x4 p0, p1;
#pragma unroll
    for (int e = 0; e < 4; ++e) p0[e] = (__bf16)lo[e], p1[e] = (__bf16)hi[e];
    bf16_t* row = dst + ((size_t)m * heads_dst + head_dst) * 128;
    *(uint2*)(row + f) = __builtin_bit_cast(uint2, p0);
    *(uint2*)(row + 64 + f) = __builtin_bit_cast(uint2, p1);
  }
}

bool gemm_supported(const GemmArgs& a, int mode) {
  if (a.m <= 0 || a.n <= 0 || a.k <= 0 || a.k % 64 != 0) return false;
  // byte offsets inside a tile's row range are 32-bit (plus the k offset of the step)
  const size_t span = (size_t)(mode == GEMM_SWIGLU ? a.n / 2 + GM_BN : GM_BN) * a.k * 2 + (size_t)a.k * 2;  // GM_BN >= BM
  if (span >= ((size_t)1 << 32)) return false;
  if (mode == GEMM_PLAIN) return a.n % 8 == 0;
  if (mode == GEMM_QKV_ROPE) return a.h_q > 0 && a.h_kv > 0 && a.n == (a.h_q + 2 * a.h_kv) * 128 && a.n % GM_BN == 0;
  if (mode == GEMM_SWIGLU) return a.n % (2 * 128) == 0 && a.n % GM_BN == 0;
  return false;
}

static std::atomic<int> g_forced_tile_rows{0};  // 0: choose per launch; 128 / 256: tests cover both tilings
void gemm_force_tile_rows(int rows) { g_forced_tile_rows.store(rows, std::memory_order_relaxed); }

// 256-row tiles unless 128-row tiles finish sooner: a launch lasts ceil(tiles / CUs) rounds of one tile each, and a
// 128-row tile costs about 0.6 of a 256-row one (half the products, less reuse of the weight fragments).
int gemm_tile_rows(const GemmArgs& a) {
  const int forced = g_forced_tile_rows.load(std::memory_order_relaxed);
  if (forced != 0) return forced;
  const int cus = device_cu_count();
  const long tiles_n = (a.n + GM_BN - 1) / GM_BN;
  const long t256 = (long)((a.m + 255) / 256) * tiles_n, t128 = (long)((a.m + 127) / 128) * tiles_n;
  const double cost256 = (double)((t256 + cus - 1) / cus), cost128 = 0.6 * (double)((t128 + cus - 1) / cus);
  return cost128 < cost256 ? 128 : 256;
}

// Contraction split: launches whose tiles would occupy at most a quarter of the CUs (few tokens against a long k:
// text chunks and decode steps through the layer, where the weights are streamed once and HBM is the bound) deal the
// k-steps to chunks, about one workgroup per CU in all, at least 4 steps per chunk, as many chunks as the scratch holds.
GemmSplit gemm_plan_split(const GemmArgs& a, int mode, size_t scratch_bytes) {
  GemmSplit p{1, a.k / GM_BK, 0};
  if (mode == GEMM_SWIGLU || scratch_bytes == 0 || gemm_uses_gemv(a)) return p;
  const int rows = gemm_tile_rows(a), cus = device_cu_count();
  const long tiles = (long)((a.m + rows - 1) / rows) * ((a.n + GM_BN - 1) / GM_BN);
  const int steps = a.k / GM_BK;
  if (tiles * 4 > cus || steps < 8) return p;
  long want = (cus + tiles - 1) / tiles;
  if (want > steps / 4) want = steps / 4;
  const size_t per_chunk = (size_t)a.m * a.n * sizeof(float);
  if ((size_t)want * per_chunk > scratch_bytes) want = (long)(scratch_bytes / per_chunk);
  if (want < 2) return p;
  p.steps_per_split = (int)((steps + want - 1) / want);
  p.split_k = (steps + p.steps_per_split - 1) / p.steps_per_split;  // every chunk non-empty
  p.scratch_bytes = (size_t)p.split_k * per_chunk;
  return p;
}

template <int MODE, int BM, int BK>
static hipError_t launch_tile(GemmArgs a, hipStream_t s) {
  static bool attr_done[QP_MAX_DEVICES] = {};
  const int dev = current_device();
  if (dev < 0) return hipErrorInvalidDevice;
  const int lds = Tile<BM, BK>::STAGES * Tile<BM, BK>::STAGE;
  if (!attr_done[dev]) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_bf16_kernel<MODE, BM, BK>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_done[dev] = true;
  }
  a.tiles_m = (a.m + BM - 1) / BM;
  a.tiles_n = (a.n + GM_BN - 1) / GM_BN;
  a.m_block = a.tiles_m < 8 ? a.tiles_m : 8;
  a.n_quads = ((a.tiles_n + 7) / 8 + 3) / 4;  // weight tiles per XCD, in fours
  const int m_chunks = (a.tiles_m + a.m_block - 1) / a.m_block;
  hipLaunchKernelGGL((gemm_bf16_kernel<MODE, BM, BK>), dim3(8 * m_chunks * a.m_block * a.n_quads * 4, a.split_k),
                     dim3(GM_NW * 64), lds, s, a);
  return hipSuccess;
}

template <int MODE>
static hipError_t launch_mode(GemmArgs a, void* scratch, size_t scratch_bytes, hipStream_t s) {
  const GemmSplit sp = gemm_plan_split(a, MODE, scratch != nullptr ? scratch_bytes : 0);
  a.split_k = sp.split_k, a.steps_per_split = sp.steps_per_split, a.partial = (float*)scratch;
  hipError_t e = gemm_tile_rows(a) == 128 ? launch_tile<MODE, 128, GM_BK>(a, s) : launch_tile<MODE, 256, GM_BK>(a, s);
  if (e != hipSuccess || a.split_k == 1) return e;
  const long threads = (long)a.m * (MODE == GEMM_QKV_ROPE ? a.n / 8 : a.n / 4);
  hipLaunchKernelGGL(gemm_reduce_kernel<MODE>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, a);
  return hipSuccess;
}

// A handful of tokens take the weight-streaming kernel (gemv_bf16.hip) unless a tiling is forced (tests then reach
// the split contraction of this kernel at those sizes too).
bool gemm_uses_gemv(const GemmArgs& a) {
  return gemv_applies(a) && g_forced_tile_rows.load(std::memory_order_relaxed) == 0;
}

hipError_t launch_gemm_bf16(const GemmArgs& a, int mode, void* scratch, size_t scratch_bytes, hipStream_t s) {
  if (gemm_uses_gemv(a)) return launch_gemv_bf16(a, mode, s);
  switch (mode) {
    case GEMM_PLAIN: return launch_mode<GEMM_PLAIN>(a, scratch, scratch_bytes, s);
    case GEMM_QKV_ROPE: return launch_mode<GEMM_QKV_ROPE>(a, scratch, scratch_bytes, s);
    case GEMM_SWIGLU: return launch_mode<GEMM_SWIGLU>(a, nullptr, 0, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace qp
