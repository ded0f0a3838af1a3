// bf16 MFMA group attention for gfx950 (head_dim 128), flash-style.
//
// What it computes (Sec. 3.2 of the paper, group-based prefill): for query head qh of KV head
// h = qh / R and group token t, softmax over {cache entries 0..C-1 of h} U {group tokens 0..t}
// of scale * q.k, times V.
//
// Mapping. The R query heads that share a KV head are stacked into one row space per KV head:
// row r = t * R + j (j = query head inside the KV group), which is also the memory order of
// Q_g[t][h*R + j][:]. A workgroup of 8 wavefronts owns 256 consecutive rows of one KV head;
// every K/V tile it stages in LDS is therefore shared by all R query heads (GQA) and by 256/R
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
// Two kernels share these building blocks:
//   attend_mfma_kernel     one barrier per tile, K/V double-buffered; every wavefront runs
//                          QK -> softmax -> PV on the same tile at the same time.
//   attend_mfma_pp_kernel  "ping-pong": the two wavefronts that share a SIMD run half a tile
//                          apart, so that one is in its matrix phase (PV of the previous tile, QK
//                          of the current one) while the other is in its softmax (VALU) phase;
//                          a workgroup barrier at every phase boundary keeps them apart. K tiles
//                          sit in a ring of 3 and V tiles in a ring of 4 LDS buffers, fetched two
//                          tiles ahead.
// Tiles beyond a wavefront's causal horizon are skipped by that wavefront; only tiles that
// straddle the diagonal (or the ragged end) are masked.
#include <stdlib.h>

#include "qp_internal.h"

namespace qp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int MF_D = 128;   // head_dim
constexpr int MF_BN = 64;   // keys per tile
constexpr int MF_KS = 272;  // LDS row stride of the K tile in bytes (256 + 16: conflict-free 16-byte reads)
constexpr int MF_VS = 288;  // LDS row stride of the V tile in bytes (256 + 32: conflict-free transposing reads)
constexpr int MF_KBYTES = MF_BN * MF_KS;
constexpr int MF_VBYTES = MF_BN * MF_VS;
constexpr int MF_NW = 8;    // wavefronts per workgroup
constexpr int MF_NT = MF_NW * 64;
constexpr int MF_BM = MF_NW * 32;               // rows per workgroup
constexpr int MF_LOADS = (MF_BN * 16) / MF_NT;  // 16-byte chunks of one tile per thread and tensor (= 2)
static_assert(MF_LOADS == 2, "tile staging below is written for two chunks per thread");

// ---- per-wavefront building blocks -------------------------------------------------------------

// S^T (64 keys x 32 rows, two 32-key blocks) = K tile . Q^T. All 16 K fragments are read before the
// first MFMA (a scheduling barrier keeps the compiler from sinking each read next to its use,
// which would serialise on LDS latency).
__device__ __forceinline__ void qk_tile(const unsigned char* kb_base, int k_off, const bf16x8 (&qf)[8],
                                        f32x16 (&st)[2]) {
  u32x4 kf[2][8];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int s = 0; s < 8; ++s) {
#if defined(QP_ABLATE) && (QP_ABLATE & 2)
      kf[kb][s] = __builtin_bit_cast(u32x4, qf[(s + kb) & 7]);
#else
      kf[kb][s] = *(const u32x4*)(kb_base + kb * 32 * MF_KS + k_off + s * 32);
#endif
    }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) st[kb][r] = 0.f;
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
      st[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[kb][s]), qf[s], st[kb], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
}

// Online softmax of one tile for this lane's row: masks keys past the row's horizon (only when
// `need_mask`), updates the running max / denominator, rescales O^T when some row's max moved,
// and leaves P^T (bf16) in the operand layout of the second product.
__device__ __forceinline__ void softmax_tile(f32x16 (&st)[2], bool need_mask, int kk0, int g, int lim_lane, float c2,
                                             float& m_run, float& l_run, f32x16 (&o)[4], bf16x8 (&pf)[4]) {
  if (need_mask) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kk = kk0 + kb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        if (kk > lim_lane) st[kb][r] = -INFINITY;
      }
  }
  // this lane: one row, 32 of the tile's 64 keys; lane^32 has the others
  float mx = st[0][0];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[kb][r]);
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float m_new = fmaxf(m_run, mx);  // finite from tile 0 on: key 0 is visible to every row
  const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
  const float mc = m_new * c2;
  float psum = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
#if defined(QP_ABLATE) && (QP_ABLATE & 1)
      const float p = fmaf(st[kb][r], c2, -mc);
#else
      const float p = __builtin_amdgcn_exp2f(fmaf(st[kb][r], c2, -mc));
#endif
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
}

// O^T (128 d x 32 rows) += V^T . P^T over the tile's 64 keys: 4 key steps of 16 x 4 d-blocks of 32.
__device__ __forceinline__ void pv_tile(const unsigned char* vb_base, int v_off, const bf16x8 (&pf)[4],
                                        f32x16 (&o)[4]) {
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
    for (int n = 0; n < 4; ++n) {
#if defined(QP_ABLATE) && (QP_ABLATE & 4)
      o[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[(ks + n) & 3], pf[ks], o[n], 0, 0, 0);
#else
      const unsigned char* p0 = vb_base + ks * 16 * MF_VS + v_off + n * 64;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0 + 8 * MF_VS));
      const s16x8 cat = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      o[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cat), pf[ks], o[n], 0, 0, 0);
#endif
    }
  }
}

// Normalise and store this lane's row of O (and its log-sum-exp).
__device__ __forceinline__ void store_row(const AttendArgs& a, const f32x16 (&o)[4], float m_run, float l_tot, float c2,
                                          int h, int r_heads, int t_lane, int j_lane, int g) {
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

// Tile staging. Prefetch registers are named scalars of a native vector type (an array of them ends
// up in scratch memory). Chunk i of a thread is 16 bytes: key (tid + 512 i) / 16 of the tile,
// d-chunk (tid + 512 i) % 16. Rows past the group's end are clamped: they are masked, never used.
#define QP_FETCH1(tile_, i_, kr_, vr_)                                                                        \
  {                                                                                                           \
    const int x = tid + MF_NT * (i_);                                                                         \
    const int kk = (tile_)*MF_BN + (x >> 4);                                                                  \
    const bool in_cache = kk < a.c;                                                                           \
    const size_t off =                                                                                        \
        (in_cache ? (size_t)kk * MF_D : (size_t)min(kk - a.c, a.n_g - 1) * gstride) + (size_t)((x & 15) * 8); \
    kr_ = *(const u32x4*)((in_cache ? ck : gk) + off);                                                        \
    vr_ = *(const u32x4*)((in_cache ? cv : gv) + off);                                                        \
  }
#define QP_FETCH(tile_)         \
  QP_FETCH1(tile_, 0, kr0, vr0) \
  QP_FETCH1(tile_, 1, kr1, vr1)
#define QP_STAGE1(kbuf_, vbuf_, i_, kr_, vr_)                    \
  {                                                              \
    const int x = tid + MF_NT * (i_);                            \
    *(u32x4*)((kbuf_) + (x >> 4) * MF_KS + (x & 15) * 16) = kr_; \
    *(u32x4*)((vbuf_) + (x >> 4) * MF_VS + (x & 15) * 16) = vr_; \
  }
#define QP_STAGE(kbuf_, vbuf_)         \
  QP_STAGE1(kbuf_, vbuf_, 0, kr0, vr0) \
  QP_STAGE1(kbuf_, vbuf_, 1, kr1, vr1)

// Common prologue of both kernels: row bookkeeping, Q fragments, source pointers, accumulators.
#define QP_ATTEND_PROLOGUE                                                                                    \
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];                                        \
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;                                              \
  const int l32 = lane & 31, g = lane >> 5;                                                                   \
  const int r_heads = a.h_q / a.h_kv;                                                                         \
  const int h = blockIdx.y;                                                                                   \
  const int n_rows = a.n_g * r_heads;                                                                         \
  const int n_rb = (n_rows + MF_BM - 1) / MF_BM;                                                              \
  const int rb = n_rb - 1 - (int)blockIdx.x; /* heaviest (latest tokens) first */                             \
  const int row0_wg = rb * MF_BM;                                                                             \
  const int row0 = row0_wg + wave * 32;                                                                       \
  const int row = row0 + l32;                                                                                 \
  const bool row_ok = row < n_rows;                                                                           \
  const int rowc = row_ok ? row : n_rows - 1;                                                                 \
  const int t_lane = rowc / r_heads;                                                                          \
  const int j_lane = rowc - t_lane * r_heads;                                                                 \
  const int lim_lane = a.c + t_lane; /* visible keys: kk <= lim_lane */                                       \
  const bf16_t* qrow = (const bf16_t*)a.q + ((size_t)t_lane * a.h_q + (size_t)h * r_heads + j_lane) * MF_D;   \
  /* horizons (wave-uniform): tokens of the first and last row of the wavefront / workgroup */               \
  const int last_row_w = min(row0 + 31, n_rows - 1);                                                          \
  const int first_row_w = min(row0, n_rows - 1);                                                              \
  const int lim_w_max = a.c + last_row_w / r_heads;                                                           \
  const int lim_w_min = a.c + first_row_w / r_heads;                                                          \
  const int last_row_wg = min(row0_wg + MF_BM - 1, n_rows - 1);                                               \
  const int n_tiles = (a.c + last_row_wg / r_heads) / MF_BN + 1;                                              \
  const bool wave_live = row0 < n_rows;                                                                       \
  /* Q^T operand: 8 k-steps of 16 d; this lane holds d = 16 s + 8 g .. + 7 of its row */                      \
  bf16x8 qf[8];                                                                                               \
  _Pragma("unroll") for (int s = 0; s < 8; ++s) qf[s] =                                                       \
      __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + 16 * s + 8 * g));                                     \
  const bf16_t* ck = (const bf16_t*)a.ck + (size_t)h * a.cap * MF_D;                                          \
  const bf16_t* cv = (const bf16_t*)a.cv + (size_t)h * a.cap * MF_D;                                          \
  const bf16_t* gk = (const bf16_t*)a.k + (size_t)h * MF_D;                                                   \
  const bf16_t* gv = (const bf16_t*)a.v + (size_t)h * MF_D;                                                   \
  const size_t gstride = (size_t)a.h_kv * MF_D;                                                               \
  u32x4 kr0, kr1, vr0, vr1;                                                                                   \
  f32x16 o[4];                                                                                                \
  _Pragma("unroll") for (int n = 0; n < 4; ++n) _Pragma("unroll") for (int r = 0; r < 16; ++r) o[n][r] = 0.f; \
  float m_run = -INFINITY; /* running row max of the raw logits q.k (unscaled) */                             \
  float l_run = 0.f;       /* this lane's share of the row's denominator */                                   \
  const float c2 = a.scale_log2;                                                                              \
  /* per-lane constant parts of the LDS read addresses */                                                     \
  const int k_off = l32 * MF_KS + g * 16;                                                                     \
  const int l16 = lane & 15, grp = lane >> 4;                                                                 \
  const int v_off = (4 * (grp >> 1) + (l16 >> 2)) * MF_VS + (16 * (grp & 1) + 4 * (l16 & 3)) * 2;

// ---- kernel 1: lock-step, double-buffered --------------------------------------------------------
__global__ __launch_bounds__(MF_NT, 2) void attend_mfma_kernel(AttendArgs a) {
  QP_ATTEND_PROLOGUE
  // LDS: [buf0: K | V][buf1: K | V]
  QP_FETCH(0)
  QP_STAGE(smem, smem + MF_KBYTES)
  __syncthreads();
#ifdef QP_TIMING
  long long tsum[6] = {0, 0, 0, 0, 0, 0};
#define QP_T(i_) { const long long now_ = clock64(); tsum[i_] += now_ - tprev; tprev = now_; }
  long long tprev = clock64();
#else
#define QP_T(i_)
#endif
  for (int tile = 0; tile < n_tiles; ++tile) {
    unsigned char* kb_base = smem + (tile & 1) * (MF_KBYTES + MF_VBYTES);
    unsigned char* nb_base = smem + ((tile & 1) ^ 1) * (MF_KBYTES + MF_VBYTES);
    if (tile + 1 < n_tiles) {
      QP_FETCH(tile + 1)
    }
    QP_T(0)
    const int kk0 = tile * MF_BN;
    if (wave_live && kk0 <= lim_w_max) {
      f32x16 st[2];
      bf16x8 pf[4];
      qk_tile(kb_base, k_off, qf, st);
      QP_T(1)
      softmax_tile(st, kk0 + MF_BN - 1 > lim_w_min, kk0, g, lim_lane, c2, m_run, l_run, o, pf);
      QP_T(2)
      pv_tile(kb_base + MF_KBYTES, v_off, pf, o);
      QP_T(3)
    }
    if (tile + 1 < n_tiles) {
      QP_STAGE(nb_base, nb_base + MF_KBYTES)
    }
    QP_T(4)
    __syncthreads();
    QP_T(5)
  }
#ifdef QP_TIMING
  if (blockIdx.x == gridDim.x / 2 && blockIdx.y == 0 && lane == 0 && a.lse != nullptr) {
    for (int i = 0; i < 6; ++i) a.lse[wave * 8 + i] = (float)tsum[i] / (float)n_tiles;
    a.lse[wave * 8 + 6] = (float)n_tiles;
  }
  if (a.lse != nullptr) return;
#endif
#undef QP_T
  if (!wave_live) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (!row_ok) return;
  store_row(a, o, m_run, l_tot, c2, h, r_heads, t_lane, j_lane, g);
}

// ---- kernel 2: direct-to-LDS staging, swizzled tiles, two key segments --------------------------------
//
// Differences from kernel 1, all aimed at the VALU work that competes with the MFMA pipe:
//   * K/V tiles go global -> LDS with global_load_lds_dwordx4 (no staging registers, no ds_write,
//     no per-chunk 64-bit address arithmetic): one instruction moves 64 lanes x 16 bytes into 1 KB of
//     LDS, lane L landing at base + 16 L. Rows are 256 bytes with no padding; bank conflicts are
//     avoided by an XOR swizzle of the 16-byte chunk index instead: K chunk c of key k sits at
//     position c ^ (k & 15), V chunk c at position c ^ ((k & 7) << 1); each lane simply fetches the
//     global chunk that belongs at its LDS position.
//   * The keys are walked as two segments, cache tiles first and then group tiles starting at group
//     token 0, so a tile never straddles the two sources and a tile's row addresses are
//     base + lane-constant (the cache's last tile and the group's diagonal tiles are masked).
//   * Tiles sit in a ring of three LDS buffers and are requested two tiles ahead, so a tile has two
//     tile-times to arrive from L2 / HBM before a wavefront waits for it.
//   * Workgroup ids are mapped so that the workgroups of one KV head run on the same XCDs (ids are
//     dealt round-robin over the 8 XCDs, each with its own L2): with 4 KV heads, XCDs 2h and 2h+1
//     serve head h, so every L2 streams one head's K/V instead of all of them.
//   * The running max is only moved when some row's max grew by more than 2^8 (the softmax
//     numerators stay below 2^8, harmless in f32/bf16), so O^T is rescaled a few times per row
//     instead of once per tile on slowly growing maxima.
//   * The row sum is taken over the bf16-rounded numerators with v_dot2c_f32_bf16 (two per
//     instruction).
constexpr int V3_TILE_BYTES = MF_BN * 256;          // one K or V tile, unpadded
constexpr int V3_STAGES = 3;                         // ring of K+V tile buffers, fetched two tiles ahead
constexpr int V3_LDS = V3_STAGES * 2 * V3_TILE_BYTES;
constexpr float V3_RESCALE_LOG2 = 8.f;

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

// 64 lanes x 16 bytes global -> LDS without passing through registers: lane L's chunk lands at
// lds_dst + 16 L (lds_dst must be wave-uniform). Written as inline assembly so that the compiler does not
// treat it as an LDS store it must wait for (vmcnt(0)) before every later LDS read; the kernel waits for
// these loads itself (s_waitcnt vmcnt) before the barrier that publishes a tile.
__device__ __forceinline__ void lds_dma16(const unsigned char* base, unsigned byte_off, unsigned char* lds_dst) {
  const unsigned lds_addr =
      __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds_dst);
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(byte_off), "s"(base), "s"(lds_addr)
      : "memory");
}

__global__ __launch_bounds__(MF_NT, 2) void attend_mfma_v3_kernel(AttendArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = a.n_g * r_heads;
  const int n_rb = (n_rows + MF_BM - 1) / MF_BM;
  // workgroup id -> (KV head, row block): ids go round-robin over the 8 XCDs
  int h, rbi;
  {
    const int wg = blockIdx.x, xcd = wg & 7, idx = wg >> 3;
    if (8 % a.h_kv == 0) {
      const int per = 8 / a.h_kv;  // XCDs per KV head
      h = xcd / per;
      rbi = idx * per + (xcd % per);
    } else if (a.h_kv % 8 == 0) {
      const int hp = a.h_kv / 8;  // KV heads per XCD
      h = (idx % hp) * 8 + xcd;
      rbi = idx / hp;
    } else {
      h = wg % a.h_kv;
      rbi = wg / a.h_kv;
    }
  }
  if (rbi >= n_rb) return;  // padding workgroups of the XCD mapping (whole workgroup, before any barrier)
  const int rb = n_rb - 1 - rbi;  // heaviest (latest tokens) first
  const int row0_wg = rb * MF_BM;
  const int row0 = row0_wg + wave * 32;
  const int row = row0 + l32;
  const bool row_ok = row < n_rows;
  const int rowc = row_ok ? row : n_rows - 1;
  const int t_lane = rowc / r_heads;
  const int j_lane = rowc - t_lane * r_heads;
  const bf16_t* qrow = (const bf16_t*)a.q + ((size_t)t_lane * a.h_q + (size_t)h * r_heads + j_lane) * MF_D;
  // wave-uniform token horizons
  const int t_w_max = min(row0 + 31, n_rows - 1) / r_heads;
  const int t_w_min = min(row0, n_rows - 1) / r_heads;
  const int t_wg_max = min(row0_wg + MF_BM - 1, n_rows - 1) / r_heads;
  const bool wave_live = row0 < n_rows;
  const int n_ct = (a.c + MF_BN - 1) / MF_BN;       // cache tiles
  const int n_tiles = n_ct + t_wg_max / MF_BN + 1;  // + group tiles

  bf16x8 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) qf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + 16 * s + 8 * g));

  const unsigned char* ck = (const unsigned char*)a.ck + (size_t)h * a.cap * (MF_D * 2);
  const unsigned char* cv = (const unsigned char*)a.cv + (size_t)h * a.cap * (MF_D * 2);
  const unsigned char* gk = (const unsigned char*)a.k + (size_t)h * (MF_D * 2);
  const unsigned char* gv = (const unsigned char*)a.v + (size_t)h * (MF_D * 2);
  const unsigned gstride_b = (unsigned)a.h_kv * (MF_D * 2);

  // staging: this wavefront's two load instructions per tensor cover keys 8*wave .. 8*wave+7 of the tile
  const int st_key0 = 8 * wave + (lane >> 4), st_key1 = st_key0 + 4;
  const int st_pos = lane & 15;
  const unsigned st_kc0 = (unsigned)((st_pos ^ (st_key0 & 15)) * 16), st_kc1 = (unsigned)((st_pos ^ (st_key1 & 15)) * 16);
  const unsigned st_vc0 = (unsigned)((st_pos ^ ((st_key0 & 7) << 1)) * 16), st_vc1 = (unsigned)((st_pos ^ ((st_key1 & 7) << 1)) * 16);
  const int st_lds = wave * 2048;  // LDS offset of this wavefront's 2 x 1 KB inside a tile

#define QP_V3_ISSUE(tile_, buf_)                                                                              \
  {                                                                                                           \
    const bool in_cache_ = (tile_) < n_ct;                                                                    \
    const int base_ = in_cache_ ? (tile_)*MF_BN : ((tile_)-n_ct) * MF_BN;                                     \
    const int last_ = in_cache_ ? a.c - 1 : a.n_g - 1; /* rows past the end are clamped: masked, never used */ \
    const unsigned stride_ = in_cache_ ? (unsigned)(MF_D * 2) : gstride_b;                                    \
    const unsigned char* ksrc_ = in_cache_ ? ck : gk;                                                         \
    const unsigned char* vsrc_ = in_cache_ ? cv : gv;                                                         \
    const unsigned r0_ = __umul24((unsigned)min(base_ + st_key0, last_), stride_);                            \
    const unsigned r1_ = __umul24((unsigned)min(base_ + st_key1, last_), stride_);                            \
    unsigned char* kdst_ = smem + (buf_) * (2 * V3_TILE_BYTES) + st_lds;                                      \
    unsigned char* vdst_ = kdst_ + V3_TILE_BYTES;                                                             \
    lds_dma16(ksrc_, r0_ + st_kc0, kdst_);                                                                    \
    lds_dma16(ksrc_, r1_ + st_kc1, kdst_ + 1024);                                                             \
    lds_dma16(vsrc_, r0_ + st_vc0, vdst_);                                                                    \
    lds_dma16(vsrc_, r1_ + st_vc1, vdst_ + 1024);                                                             \
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

  f32x16 o[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[n][r] = 0.f;
  float m_run = -INFINITY;  // reference max of the raw logits (lags the true running max by < 2^8 after scaling)
  float l_run = 0.f;        // this lane's share of the row's denominator
  const float c2 = a.scale_log2;
  const float lazy = V3_RESCALE_LOG2 / c2;
  bf16x2 ones;
  ones[0] = (__bf16)1.0f;
  ones[1] = (__bf16)1.0f;

  // The Q fragments must have arrived before the first tile request: from here on the only vector-memory
  // operations in flight are the tile requests, which the compiler does not see (it would otherwise
  // re-wait for "pending" Q loads inside the loop and drain the tile requests with them).
  __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
  // each wavefront has 4 loads in flight per requested tile; vmcnt(4) = everything but the newest tile has landed
  QP_V3_ISSUE(0, 0)
  if (n_tiles > 1) {
    QP_V3_ISSUE(1, 1)
    __builtin_amdgcn_s_waitcnt(0x0f74);  // vmcnt(4)
  } else {
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
  }
  __syncthreads();

  int buf = 0, buf_next2 = 2;  // ring positions of tile and tile + 2
  for (int tile = 0; tile < n_tiles; ++tile) {
#if !(defined(QP_ABLATE) && (QP_ABLATE & 8))
    // buffer of tile+2 = buffer of tile-1: every wavefront finished reading it before the last barrier
    if (tile + 2 < n_tiles) QP_V3_ISSUE(tile + 2, buf_next2)
#endif
    // visibility inside this tile: key_local <= lim_local
    const bool in_cache = tile < n_ct;
    const int gt0 = (tile - n_ct) * MF_BN;  // first group token of a group tile
    const bool live = wave_live && (in_cache || gt0 <= t_w_max);
    if (live) {
      const int lim_local = in_cache ? a.c - 1 - tile * MF_BN : t_lane - gt0;
      const bool need_mask = in_cache ? (a.c - tile * MF_BN < MF_BN) : (gt0 + MF_BN - 1 > t_w_min);
      const unsigned char* kt = smem + buf * (2 * V3_TILE_BYTES);
      const unsigned char* vt = kt + V3_TILE_BYTES;
      // ---- S^T = K . Q^T
      f32x16 st[2];
      {
        u32x4 kf[2][8];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int s = 0; s < 8; ++s) {
#if defined(QP_ABLATE) && (QP_ABLATE & 2)
            kf[kb][s] = __builtin_bit_cast(u32x4, qf[(s + kb) & 7]);
#else
            kf[kb][s] = *(const u32x4*)(kt + kb * 32 * 256 + k_addr[s]);
#endif
          }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) st[kb][r] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
          for (int kb = 0; kb < 2; ++kb) {
#if defined(QP_ABLATE) && (QP_ABLATE & 64)
            st[kb][s] += __builtin_bit_cast(float, kf[kb][s][0]);
#else
            st[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[kb][s]), qf[s], st[kb], 0, 0, 0);
#endif
          }
        __builtin_amdgcn_sched_barrier(0);
      }
      // ---- softmax
#if defined(QP_ABLATE) && (QP_ABLATE & 32)
      bf16x8 pf[4];
      for (int i = 0; i < 4; ++i) { u32x4 t_ = __builtin_bit_cast(u32x4, qf[i]); t_[0] ^= __builtin_bit_cast(unsigned, st[i & 1][i]); t_[1] ^= __builtin_bit_cast(unsigned, st[i & 1][i + 4]); t_[2] ^= __builtin_bit_cast(unsigned, st[i & 1][i + 8]); t_[3] ^= __builtin_bit_cast(unsigned, st[i & 1][i + 12]); pf[i] = __builtin_bit_cast(bf16x8, t_); }
      (void)lim_local; (void)need_mask; (void)lazy; (void)ones;
#else
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
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // first tile: m_run = -inf, so the max is adopted; key 0 is visible to every row, so it is finite
      const float m_new = (mx > m_run + lazy) ? mx : m_run;
      const float mc = m_new * c2;
      bf16x8 pf[4];
      float psum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          bf16x2 pr;
#if defined(QP_ABLATE) && (QP_ABLATE & 1)
          pr[0] = (__bf16)(fmaf(st[kb][r], c2, -mc));
          pr[1] = (__bf16)(fmaf(st[kb][r + 1], c2, -mc));
#else
          pr[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(st[kb][r], c2, -mc));
          pr[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(st[kb][r + 1], c2, -mc));
#endif
          psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
          pf[kb * 2 + (r >> 3)][r & 7] = pr[0];
          pf[kb * 2 + (r >> 3)][(r & 7) + 1] = pr[1];
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
#endif
      // ---- O^T += V^T . P^T
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int n = 0; n < 4; ++n) {
#if defined(QP_ABLATE) && (QP_ABLATE & 128)
          o[n][ks] += (float)pf[ks][n];
#elif defined(QP_ABLATE) && (QP_ABLATE & 4)
          o[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[(ks + n) & 3], pf[ks], o[n], 0, 0, 0);
#else
          const unsigned char* p0 = vt + ks * 16 * 256 + v_addr[n];
          s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
          s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0 + 8 * 256));
          const s16x8 cat = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cat), pf[ks], o[n], 0, 0, 0);
#endif
        }
      }
    }
#if !(defined(QP_ABLATE) && (QP_ABLATE & 16))
    // this wavefront's part of the next tile has landed in LDS (the tile after it may still be in flight)
    if (tile + 2 < n_tiles) __builtin_amdgcn_s_waitcnt(0x0f74);  // vmcnt(4)
    else __builtin_amdgcn_s_waitcnt(0x0f70);                     // vmcnt(0)
    __syncthreads();
#endif
    buf = buf == V3_STAGES - 1 ? 0 : buf + 1;
    buf_next2 = buf_next2 == V3_STAGES - 1 ? 0 : buf_next2 + 1;
  }
#undef QP_V3_ISSUE

  if (!wave_live) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (!row_ok) return;
  store_row(a, o, m_run, l_tot, c2, h, r_heads, t_lane, j_lane, g);
}

bool attend_mfma_supported(const AttendArgs& a, int dtype) {
  // 24-bit row and 32-bit byte offsets inside one head's cache / the group's K, V
  return dtype == QP_BF16 && a.d == MF_D && a.h_kv <= 65535 && (long long)a.cap * (MF_D * 2) < (1ll << 31) &&
         (long long)a.n_g * a.h_kv * (MF_D * 2) < (1ll << 31) && a.cap < (1 << 24);
}

void launch_attend_mfma(const AttendArgs& a, hipStream_t s) {
  static int variant = -1;
  if (variant < 0) {
    const char* e = getenv("QP_MFMA_VARIANT");
    variant = e ? atoi(e) : 3;
    (void)hipFuncSetAttribute((const void*)attend_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                              2 * (MF_KBYTES + MF_VBYTES));
    (void)hipFuncSetAttribute((const void*)attend_mfma_v3_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, V3_LDS);
  }
  const int n_rows = a.n_g * (a.h_q / a.h_kv);
  const int n_rb = (n_rows + MF_BM - 1) / MF_BM;
  if (variant == 4) {
    launch_attend_mfma64(a, s);
    return;
  }
  if (variant == 3) {
    int n_wg = n_rb * a.h_kv;
    if (8 % a.h_kv == 0) {
      const int per = 8 / a.h_kv;
      n_wg = (n_rb + per - 1) / per * 8;
    }
    hipLaunchKernelGGL(attend_mfma_v3_kernel, dim3(n_wg), dim3(MF_NT), V3_LDS, s, a);
  }
  else
    hipLaunchKernelGGL(attend_mfma_kernel, dim3(n_rb, a.h_kv), dim3(MF_NT), 2 * (MF_KBYTES + MF_VBYTES), s, a);
}

#undef QP_FETCH
#undef QP_FETCH1
#undef QP_STAGE
#undef QP_STAGE1
#undef QP_ATTEND_PROLOGUE

}  // namespace qp
