// bf16 MFMA group attention for gfx950 (head_dim 128), flash-style.
//
// What it computes (Sec. 3.2 of the paper, group-based prefill): for query head qh of KV head
// h = qh / R and group token t, softmax over {cache entries 0..C-1 of h} U {group tokens 0..t}
// of scale * q.k, times V.
//
// Mapping. The R query heads that share a KV head are stacked into one row space per KV head:
// row r = t * R + j (j = query head inside the KV group), which is also the memory order of
// Q_g[t][h*R + j][:]. A workgroup of 8 wavefronts owns 256 rows of one KV head; every K/V tile it
// stages in LDS is shared by all R query heads (GQA). Two row mappings, chosen by the launcher:
//   * more workgroups than CUs: 256 consecutive rows each, latest tokens (longest key range) first,
//     so that the short workgroups fill the tail of the launch;
//   * at most one workgroup per CU (all resident at once, the launch lasts as long as its longest
//     workgroup): two half blocks of 128 consecutive rows each, one from the early end of the group
//     and its mirror from the late end, so that all workgroups carry the same causal work.
// The keys are walked as two segments, cache tiles first and then group tiles starting
// at group token 0, so a tile never straddles the two sources; only the cache's last tile and the
// group's diagonal tiles are masked, and a wavefront skips group tiles beyond its causal horizon.
// Key split: the cache tiles of a row block can be dealt to several workgroups (chunks), each leaving a normalised
// partial output and its log-sum-exp for a merge launch. The planner splits every row block when few rows meet a
// long cache (so that the launch covers the chip), and, in launches of several rounds of workgroups, only the row
// blocks of a partly filled last round (so that their chunks fill the compute units evenly); see plan_attend_mfma.
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
// Choices aimed at the vector/LDS work that competes with the matrix pipe:
//   * K/V tiles go global -> LDS with global_load_lds_dwordx4 (no staging registers, no ds_write):
//     one instruction moves 64 lanes x 16 bytes into 1 KB of LDS, lane L landing at base + 16 L.
//     Rows are 256 bytes, unpadded; bank conflicts are avoided by an XOR swizzle of the 16-byte
//     chunk index: K chunk c of key k sits at position c ^ (k & 15), V chunk c at position
//     c ^ ((k & 7) << 1); each lane fetches the global chunk that belongs at its LDS position.
//   * Tiles sit in a ring of LDS buffers and are requested two tiles ahead.
//   * Workgroup ids are mapped so that the workgroups of one KV head run on the same XCDs (ids are
//     dealt round-robin over the 8 XCDs, each with its own L2): with 4 KV heads, XCDs 2h and 2h+1
//     serve head h, so every L2 streams one head's K/V instead of all of them.
//   * The reference max only moves when some row's max grew by more than 2^8 (the softmax
//     numerators stay below 2^8, harmless in f32/bf16), so O^T is rescaled a few times per row
//     instead of once per tile on slowly growing maxima.
//   * The row sum is taken over the bf16-rounded numerators with v_dot2c_f32_bf16.
// Schedule: every wavefront runs QK -> softmax -> PV on the same tile, one barrier per tile. Schedules that
// keep the two wavefronts of a SIMD half a tile apart (one in its matrix phase while the other is in its
// softmax phase: with a barrier per phase, or with opposite phase order between two barriers), software
// pipelining inside a wavefront, and raising the wavefront's priority (s_setprio) around the matrix phases
// or around the softmax were all measured and were all slower than this plain loop (1-19 %); two tiles per
// barrier (a ring of four slots, so that the two wavefronts of a SIMD drift apart between barriers) measured the
// same within 2 %. At full occupancy the chip lowers its clock under this kernel: time per tile is then set by
// the energy a tile costs, not by how well the phases overlap.
#include "qp_internal.h"

#include <algorithm>

namespace qp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int MF_D = 128;               // head_dim
constexpr int MF_BN = 64;               // keys per tile
constexpr int MF_NW = 8;                // wavefronts per workgroup
constexpr int MF_NT = MF_NW * 64;
constexpr int MF_HB = MF_NW / 2 * 32;   // rows per half block (4 wavefronts); a workgroup owns two half blocks
constexpr int MF_TILE = MF_BN * 256;    // bytes of one K or V tile (unpadded, swizzled)
constexpr int MF_SLOT = 2 * MF_TILE;    // K tile + V tile
constexpr int MF_STAGES = 3;            // ring of K+V tile slots
constexpr float MF_RESCALE_LOG2 = 8.f;  // move the reference max only when it grows by more than 2^8
constexpr int MF_VMCNT0 = 0x0f70;       // s_waitcnt vmcnt(0), other counters untouched
constexpr int MF_VMCNT4 = 0x0f74;       // s_waitcnt vmcnt(4)
constexpr int MF_SPLIT_BELOW = 128;     // launches of fewer workgroups split the cache over chunks
constexpr int MF_MAX_SPLIT = 128;       // chunks at most
constexpr size_t MF_SPLIT_ALL_BYTES = (size_t)32 << 20;  // scratch that a split of every row block takes at most
constexpr int MF_TAIL_SPLIT_MAX = 8;    // chunks per row block when only the last round's row blocks are split
constexpr int MF_TAIL_MIN_TILES = 16;   // ... whose chunks hold at least this many cache tiles

// S^T (64 keys x 32 rows, two 32-key blocks) = K tile . Q^T. All 16 K fragments are read before the
// first MFMA (a scheduling barrier keeps the compiler from sinking each read next to its use,
// which would serialise on LDS latency).
__device__ __forceinline__ void qk_tile(const unsigned char* kt, const int (&k_addr)[8], const bf16x8 (&qf)[8],
                                        f32x16 (&st)[2]) {
  u32x4 kf[2][8];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int s = 0; s < 8; ++s) kf[kb][s] = *(const u32x4*)(kt + kb * 32 * 256 + k_addr[s]);
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

// Online softmax of one tile for this lane's row (32 of the tile's 64 keys; lane ^ 32 has the others):
// masks keys with key_local > lim_local (only when need_mask), updates the reference max / the lane's
// share of the denominator, rescales O^T when the reference moved, leaves P^T (bf16) in pf.
__device__ __forceinline__ void softmax_tile(f32x16 (&st)[2], bool need_mask, int lim_local, int g, float c2,
                                             float lazy, float& m_run, float& l_run, f32x16 (&o)[4],
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
  mx = max_halves(mx);
  // first tile: m_run = -inf, so the max is adopted; key 0 is visible to every row, so it is finite
  const float m_new = (mx > m_run + lazy) ? mx : m_run;
  const float mc = m_new * c2;
  bf16x2 ones;
  ones[0] = (__bf16)1.0f;
  ones[1] = (__bf16)1.0f;
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

// O^T (128 d x 32 rows) += V^T . P^T over the tile's 64 keys: 4 key steps of 16 x 4 d-blocks of 32.
__device__ __forceinline__ void pv_tile(const unsigned char* vt, const int (&v_addr)[4], const bf16x8 (&pf)[4],
                                        f32x16 (&o)[4]) {
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      const unsigned char* p0 = vt + ks * 16 * 256 + v_addr[n];
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0 + 8 * 256));
      const s16x8 cat = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      o[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cat), pf[ks], o[n], 0, 0, 0);
    }
  }
}

// F8: the cache's K~ and V~ hold one E4M3 byte per element (the pruned cache's 8-bit format). Their tiles cannot go
// global -> LDS directly: every wavefront loads its share of a tile into registers one tile ahead (8 bytes per lane
// and row), widens it exactly to bf16 and writes it to the ring slot in the same swizzled layout, so that everything
// after the staging is the same code. The group's own tiles are bf16 and staged as usual.
template <bool F8>
__global__ __launch_bounds__(MF_NT, 2) void attend_mfma_kernel(AttendArgs a) {
  constexpr int STAGES = MF_STAGES;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform for the compiler too: scalar address and branch work
  const int l32 = lane & 31, g = lane >> 5;
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = a.n_g * r_heads;
  const int n_hb = (n_rows + MF_HB - 1) / MF_HB;  // half blocks of 128 rows
  const int n_rb = (n_hb + 1) / 2;                // workgroups per KV head (256 rows or a pair of half blocks)
  // Work items of a KV head: the row blocks that one workgroup serves whole (longest first), then the chunks of the
  // split row blocks (the shortest ones), chunk by chunk.
  const int n_whole = n_rb - (a.n_split > 1 ? a.split_rb : 0);
  const int n_items = n_whole + (n_rb - n_whole) * a.n_split;
  // workgroup id -> (KV head, item): ids go round-robin over the 8 XCDs
  int h, item;
  {
    const int wg = blockIdx.x, xcd = wg & 7, idx = wg >> 3;
    if (8 % a.h_kv == 0) {
      const int per = 8 / a.h_kv;  // XCDs per KV head
      h = xcd / per;
      item = idx * per + (xcd % per);
    } else if (a.h_kv % 8 == 0) {
      const int hp = a.h_kv / 8;  // KV heads per XCD
      h = (idx % hp) * 8 + xcd;
      item = idx / hp;
    } else {
      h = wg % a.h_kv;
      item = wg / a.h_kv;
    }
  }
  if (item >= n_items) return;    // padding workgroups of the XCD mapping (whole workgroup, before any barrier)
  int rbi = item, chunk = 0, my_split = 1;  // row block (0 = latest tokens), key chunk, chunks of this row block
  if (item >= n_whole) {
    const int e = item - n_whole, n_sp = n_rb - n_whole;
    chunk = e / n_sp;
    rbi = n_whole + (e - chunk * n_sp);
    my_split = a.n_split;
  }
  // Mirrored mapping: the workgroup owns half block rbi (early tokens, short key range) and its mirror
  // n_hb-1-rbi (late tokens, long key range). Wavefronts 0..3 take the early half block and 4..7 the late one:
  // wavefronts w and w+4 share a SIMD, so each SIMD keeps one wavefront busy after the early rows have reached
  // their causal horizon. Consecutive mapping: half blocks 2 rb and 2 rb + 1 with rb counted from the late end.
  const int half = wave >> 2;
  const int hb_late = a.mirrored ? n_hb - 1 - rbi : min(2 * (n_rb - 1 - rbi) + 1, n_hb - 1);
  const int hb_early = a.mirrored ? rbi : 2 * (n_rb - 1 - rbi);
  const int hb = half ? hb_late : hb_early;
  const bool unpaired = half == 0 && hb_early == hb_late;  // odd count: that half block is served as "late" only
  const int row0 = hb * MF_HB + (wave & 3) * 32;
  const int row = row0 + l32;
  const bool row_ok = row < n_rows;
  const int rowc = row_ok ? row : n_rows - 1;
  const int t_lane = rowc / r_heads;
  const int j_lane = rowc - t_lane * r_heads;
  const bf16_t* qrow = (const bf16_t*)a.q + ((size_t)t_lane * a.h_q + (size_t)h * r_heads + j_lane) * MF_D;
  // wave-uniform token horizons
  const int t_w_max = min(row0 + 31, n_rows - 1) / r_heads;
  const int t_w_min = min(row0, n_rows - 1) / r_heads;
  const int t_wg_max = min(hb_late * MF_HB + MF_HB - 1, n_rows - 1) / r_heads;
  const bool wave_live = row0 < n_rows && !unpaired;
  const int n_ct = (a.c + MF_BN - 1) / MF_BN;       // cache tiles
  const int n_tiles = n_ct + t_wg_max / MF_BN + 1;  // + group tiles
  // key split: a chunk walks cache tiles [t_begin, t_end); the last chunk goes on through the group tiles
  const int t_begin = chunk * a.split_tiles;
  const int t_end = chunk == my_split - 1 ? n_tiles : t_begin + a.split_tiles;

  constexpr int CROW = F8 ? MF_D : MF_D * 2;  // bytes of one cached row
  const unsigned char* ck = (const unsigned char*)a.ck + (size_t)h * a.cap * CROW;
  const unsigned char* cv = (const unsigned char*)a.cv + (size_t)h * a.cap * CROW;
  const unsigned char* gk = (const unsigned char*)a.k + (size_t)h * (MF_D * 2);
  const unsigned char* gv = (const unsigned char*)a.v + (size_t)h * (MF_D * 2);
  const unsigned gstride_b = (unsigned)a.h_kv * (MF_D * 2);

  // staging: this wavefront's two load instructions per tensor cover keys 8*wave .. 8*wave+7 of the tile;
  // LDS position (lane & 15) of key row (lane >> 4) <- the global chunk position ^ swizzle(key)
  const int st_key0 = 8 * wave + (lane >> 4), st_key1 = st_key0 + 4;
  const int st_pos = lane & 15;
  const unsigned st_kc0 = (unsigned)((st_pos ^ (st_key0 & 15)) * 16), st_kc1 = (unsigned)((st_pos ^ (st_key1 & 15)) * 16);
  const unsigned st_vc0 = (unsigned)((st_pos ^ ((st_key0 & 7) << 1)) * 16),
                 st_vc1 = (unsigned)((st_pos ^ ((st_key1 & 7) << 1)) * 16);
  const int st_lds = wave * 2048;  // LDS offset of this wavefront's 2 x 1 KB inside a tile

  // request tile `tile_` into ring slot `slot_` (4 loads per wavefront)
#define QP_ISSUE(tile_, slot_)                                                                                 \
  {                                                                                                            \
    const bool in_cache_ = (tile_) < n_ct;                                                                     \
    const int base_ = in_cache_ ? (tile_)*MF_BN : ((tile_)-n_ct) * MF_BN;                                      \
    const int last_ = in_cache_ ? a.c - 1 : a.n_g - 1; /* rows past the end are clamped: masked, never used */ \
    const unsigned stride_ = in_cache_ ? (unsigned)(MF_D * 2) : gstride_b;                                     \
    const unsigned char* ksrc_ = in_cache_ ? ck : gk;                                                          \
    const unsigned char* vsrc_ = in_cache_ ? cv : gv;                                                          \
    const unsigned r0_ = __umul24((unsigned)min(base_ + st_key0, last_), stride_);                             \
    const unsigned r1_ = __umul24((unsigned)min(base_ + st_key1, last_), stride_);                             \
    unsigned char* kdst_ = smem + (slot_)*MF_SLOT + st_lds;                                                    \
    unsigned char* vdst_ = kdst_ + MF_TILE;                                                                    \
    lds_dma16(ksrc_, r0_ + st_kc0, kdst_);                                                                     \
    lds_dma16(ksrc_, r1_ + st_kc1, kdst_ + 1024);                                                              \
    lds_dma16(vsrc_, r0_ + st_vc0, vdst_);                                                                     \
    lds_dma16(vsrc_, r1_ + st_vc1, vdst_ + 1024);                                                              \
  }

  // 8-bit cache tiles: this lane's 8-byte pieces of the pending tile (same keys and LDS positions as above; global
  // chunk c of a row is 8 bytes at c * 8), and their widened form written to a ring slot
  uint2 f8k0 = make_uint2(0, 0), f8k1 = f8k0, f8v0 = f8k0, f8v1 = f8k0;
  auto f8_load = [&](int tile_) {
    const int base_ = tile_ * MF_BN, last_ = a.c - 1;
    const unsigned r0_ = (unsigned)min(base_ + st_key0, last_) * (unsigned)MF_D;
    const unsigned r1_ = (unsigned)min(base_ + st_key1, last_) * (unsigned)MF_D;
    f8k0 = *(const uint2*)(ck + r0_ + (st_kc0 >> 1));
    f8k1 = *(const uint2*)(ck + r1_ + (st_kc1 >> 1));
    f8v0 = *(const uint2*)(cv + r0_ + (st_vc0 >> 1));
    f8v1 = *(const uint2*)(cv + r1_ + (st_vc1 >> 1));
  };
  auto widen8 = [](uint2 p) -> u32x4 {  // 8 E4M3 bytes -> 8 bf16 (the f32 values are exact; their high halves are the bf16)
    const auto a0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)p.x, false), a1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)p.x, true);
    const auto b0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)p.y, false), b1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)p.y, true);
    u32x4 o;
    o.x = (__float_as_uint(a0[0]) >> 16) | (__float_as_uint(a0[1]) & 0xffff0000u);
    o.y = (__float_as_uint(a1[0]) >> 16) | (__float_as_uint(a1[1]) & 0xffff0000u);
    o.z = (__float_as_uint(b0[0]) >> 16) | (__float_as_uint(b0[1]) & 0xffff0000u);
    o.w = (__float_as_uint(b1[0]) >> 16) | (__float_as_uint(b1[1]) & 0xffff0000u);
    return o;
  };
  auto f8_store = [&](int slot_) {
    unsigned char* kdst_ = smem + slot_ * MF_SLOT + st_lds + lane * 16;
    unsigned char* vdst_ = kdst_ + MF_TILE;
    *(u32x4*)(kdst_) = widen8(f8k0);
    *(u32x4*)(kdst_ + 1024) = widen8(f8k1);
    *(u32x4*)(vdst_) = widen8(f8v0);
    *(u32x4*)(vdst_ + 1024) = widen8(f8v1);
  };
  // stage tile `tile_` for slot `slot_`: cache tiles of an 8-bit cache go through registers (f8_store follows later)
#define QP_STAGE(tile_, slot_)                    \
  {                                               \
    if (F8 && (tile_) < n_ct) f8_load(tile_);     \
    else QP_ISSUE(tile_, slot_)                   \
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
  const float lazy = MF_RESCALE_LOG2 / c2;

  // visibility of tile `tile_` for this wavefront / lane
#define QP_TILE_VIEW(tile_)                                                                             \
  const bool in_cache = (tile_) < n_ct;                                                                 \
  const int gt0 = ((tile_)-n_ct) * MF_BN; /* first group token of a group tile */                       \
  const bool live = wave_live && (in_cache || gt0 <= t_w_max);                                          \
  const int lim_local = in_cache ? a.c - 1 - (tile_)*MF_BN : t_lane - gt0; /* key_local <= lim_local */ \
  const bool need_mask = in_cache ? (a.c - (tile_)*MF_BN < MF_BN) : (gt0 + MF_BN - 1 > t_w_min);

  // each wavefront has 4 loads in flight per requested tile: vmcnt(4) = all but the newest tile have landed
  QP_STAGE(t_begin, 0)
  if (F8 && t_begin < n_ct) f8_store(0);
  if (t_begin + 1 < t_end) {
    QP_STAGE(t_begin + 1, 1)
    if (F8 && t_begin + 1 < n_ct) f8_store(1);
  }
  // Q^T operand: 8 k-steps of 16 d; this lane holds d = 16 s + 8 g .. + 7 of its row. Requested behind the first
  // tiles so that the two latencies overlap (short key chunks are mostly prologue).
  bf16x8 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) qf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + 16 * s + 8 * g));
  // The Q fragments must have arrived before the loop: from there on the only vector-memory operations in flight
  // are the tile requests, which the compiler does not see (it would otherwise re-wait for "pending" Q loads
  // inside the loop and drain the tile requests with them).
  __builtin_amdgcn_s_waitcnt(MF_VMCNT0);
  __syncthreads();

  {
    int slot = 0, slot2 = 2;  // ring positions of tile and tile + 2
    for (int tile = t_begin; tile < t_end; ++tile) {
      // slot of tile+2 = slot of tile-1: every wavefront finished reading it before the last barrier
      if (tile + 2 < t_end) QP_STAGE(tile + 2, slot2)
      QP_TILE_VIEW(tile)
      if (live) {
        const unsigned char* kt = smem + slot * MF_SLOT;
        f32x16 st[2];
        bf16x8 pf[4];
        qk_tile(kt, k_addr, qf, st);
        softmax_tile(st, need_mask, lim_local, g, c2, lazy, m_run, l_run, o, pf);
        pv_tile(kt + MF_TILE, v_addr, pf, o);
      }
      if (F8) {
        // the pending 8-bit tile was requested a whole tile ago: widen it into its slot (last read before the
        // previous barrier); every request, direct ones included, is awaited here
        if (tile + 2 < t_end && tile + 2 < n_ct) f8_store(slot2);
        __builtin_amdgcn_s_waitcnt(MF_VMCNT0);
      } else {
        // this wavefront's part of the next tile has landed in LDS (the tile after it may still be in flight)
        if (tile + 2 < t_end) __builtin_amdgcn_s_waitcnt(MF_VMCNT4);
        else __builtin_amdgcn_s_waitcnt(MF_VMCNT0);
      }
      __syncthreads();
      slot = slot == STAGES - 1 ? 0 : slot + 1;
      slot2 = slot2 == STAGES - 1 ? 0 : slot2 + 1;
    }
  }
#undef QP_STAGE
#undef QP_ISSUE
#undef QP_TILE_VIEW

  if (!wave_live) return;
  const float l_tot = sum_halves(l_run);
  if (!row_ok) return;
  const float inv = 1.f / l_tot;
  if (my_split > 1) {
    // partial result of this chunk: every chunk starts on a cache tile, whose keys all rows see, so l_tot > 0
    const size_t prow = (size_t)chunk * ((size_t)a.h_kv * a.part_rows) + (size_t)h * a.part_rows + row;
    float* po = a.part_o + prow * MF_D;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        *(float4*)(po + 32 * n + 8 * q4 + 4 * g) = make_float4(o[n][4 * q4] * inv, o[n][4 * q4 + 1] * inv,
                                                               o[n][4 * q4 + 2] * inv, o[n][4 * q4 + 3] * inv);
    if (g == 0) a.part_lse[prow] = m_run * c2 + log2f(l_tot);
    return;
  }
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

// Merge of the key split: out[row] = sum_c 2^(lse_c - lse) O_c[row], lse = log2 sum_c 2^lse_c. One workgroup of 8
// wavefronts per row: wavefront w takes chunks w, w+8, ..., eight at a time with all their loads in flight at once
// (the log-sum-exps and the partial rows alike, so a wavefront pays one memory round trip per batch), merges them
// around its own maximum, and the eight results meet in LDS. Lane l owns d = 2l, 2l+1.
constexpr int MG_WAVES = 8;
__global__ __launch_bounds__(MG_WAVES * 64) void attend_merge_kernel(AttendArgs a) {
  __shared__ float red[MG_WAVES][64][2], red_m[MG_WAVES], red_l[MG_WAVES];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = a.part_rows;  // rows per KV head that were split
  const long total = (long)a.h_kv * n_rows;
  const long grow = blockIdx.x;
  const int h = (int)(grow / n_rows), row = (int)(grow - (long)h * n_rows);
  const int t = row / r_heads, j = row - t * r_heads;
  float m = -INFINITY, den = 0.f, acc0 = 0.f, acc1 = 0.f;  // this wavefront's chunks, relative to m
  for (int c0 = wave; c0 < a.n_split; c0 += 8 * MG_WAVES) {
    float ls[8];
    float2 po[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int c = min(c0 + MG_WAVES * u, a.n_split - 1);
      ls[u] = c0 + MG_WAVES * u < a.n_split ? a.part_lse[(size_t)c * total + grow] : -INFINITY;
      po[u] = *(const float2*)(a.part_o + ((size_t)c * total + grow) * MF_D + 2 * lane);
    }
    float mb = ls[0];  // finite: chunk c0 exists
#pragma unroll
    for (int u = 1; u < 8; ++u) mb = fmaxf(mb, ls[u]);
    const float m_new = fmaxf(m, mb);
    const float keep = exp2f(m - m_new);  // 0 the first time
    den *= keep;
    acc0 *= keep;
    acc1 *= keep;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float w = exp2f(ls[u] - m_new);
      den += w;
      acc0 = fmaf(w, po[u].x, acc0);
      acc1 = fmaf(w, po[u].y, acc1);
    }
    m = m_new;
  }
  red[wave][lane][0] = acc0;
  red[wave][lane][1] = acc1;
  if (lane == 0) {
    red_m[wave] = m;  // -inf for a wavefront without chunks: weight 0 below
    red_l[wave] = den;
  }
  __syncthreads();
  if (wave != 0) return;
  float big = red_m[0];
#pragma unroll
  for (int w = 1; w < MG_WAVES; ++w) big = fmaxf(big, red_m[w]);
  float dsum = 0.f, o0 = 0.f, o1 = 0.f;
#pragma unroll
  for (int w = 0; w < MG_WAVES; ++w) {
    const float wgt = exp2f(red_m[w] - big);
    dsum = fmaf(wgt, red_l[w], dsum);
    o0 = fmaf(wgt, red[w][lane][0], o0);
    o1 = fmaf(wgt, red[w][lane][1], o1);
  }
  const float inv = 1.f / dsum;
  bf16x2 pk;
  pk[0] = (__bf16)(o0 * inv);
  pk[1] = (__bf16)(o1 * inv);
  bf16_t* orow = (bf16_t*)a.out + ((size_t)t * a.h_q + (size_t)h * r_heads + j) * MF_D;
  *(uint32_t*)(orow + 2 * lane) = __builtin_bit_cast(uint32_t, pk);
  if (a.lse != nullptr && lane == 0)
    a.lse[(size_t)(h * r_heads + j) * a.n_g + t] = (big + log2f(dsum)) * 0.6931471805599453f;
}

// The same merge for launches of many rows and few chunks (small groups against a long cache: thousands of rows,
// a handful of chunks): one wavefront per row, four rows per workgroup, no exchange through LDS. Same arithmetic
// order per row as a single wavefront of attend_merge_kernel would use: chunks in batches of 8 around a running max.
constexpr int MR_WAVES = 4;
__global__ __launch_bounds__(MR_WAVES * 64) void attend_merge_rows_kernel(AttendArgs a) {
  const int lane = threadIdx.x & 63;
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = a.part_rows;  // rows per KV head that were split
  const long total = (long)a.h_kv * n_rows;
  const long grow = (long)blockIdx.x * MR_WAVES + (threadIdx.x >> 6);
  if (grow >= total) return;
  const int h = (int)(grow / n_rows), row = (int)(grow - (long)h * n_rows);
  const int t = row / r_heads, j = row - t * r_heads;
  float m = -INFINITY, den = 0.f, acc0 = 0.f, acc1 = 0.f;
  for (int c0 = 0; c0 < a.n_split; c0 += 8) {
    float ls[8];
    float2 po[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int c = min(c0 + u, a.n_split - 1);
      ls[u] = c0 + u < a.n_split ? a.part_lse[(size_t)c * total + grow] : -INFINITY;
      po[u] = *(const float2*)(a.part_o + ((size_t)c * total + grow) * MF_D + 2 * lane);
    }
    float mb = ls[0];  // finite: chunk c0 exists
#pragma unroll
    for (int u = 1; u < 8; ++u) mb = fmaxf(mb, ls[u]);
    const float m_new = fmaxf(m, mb);
    const float keep = exp2f(m - m_new);  // 0 the first time
    den *= keep;
    acc0 *= keep;
    acc1 *= keep;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float w = exp2f(ls[u] - m_new);
      den += w;
      acc0 = fmaf(w, po[u].x, acc0);
      acc1 = fmaf(w, po[u].y, acc1);
    }
    m = m_new;
  }
  const float inv = 1.f / den;
  bf16x2 pk;
  pk[0] = (__bf16)(acc0 * inv);
  pk[1] = (__bf16)(acc1 * inv);
  bf16_t* orow = (bf16_t*)a.out + ((size_t)t * a.h_q + (size_t)h * r_heads + j) * MF_D;
  *(uint32_t*)(orow + 2 * lane) = __builtin_bit_cast(uint32_t, pk);
  if (a.lse != nullptr && lane == 0)
    a.lse[(size_t)(h * r_heads + j) * a.n_g + t] = (m + log2f(den)) * 0.6931471805599453f;
}

bool attend_mfma_supported(const AttendArgs& a, int dtype) {
  // 24-bit row and 32-bit byte offsets inside one head's cache / the group's K, V
  return dtype == QP_BF16 && a.d == MF_D && a.h_kv <= 65535 && (long long)a.cap * (MF_D * 2) < (1ll << 31) &&
         (long long)a.n_g * a.h_kv * (MF_D * 2) < (1ll << 31) && a.cap < (1 << 24);
}

// Chunk length (cache tiles) for `want` chunks of a row block whose rows see at most n_gt group tiles: the last chunk
// also walks those, so chunks are made just long enough that its cache tiles plus the group tiles do not exceed the
// others' length by more than one tile (all chunks end together). Every chunk starts on a cache tile.
static int chunk_tiles(int n_ct, int want, int n_gt) {
  int st = (n_ct + want - 1) / want;
  while (st < n_ct - 1 && n_ct - ((n_ct + st - 1) / st - 1) * st + n_gt > st + 1) ++st;
  return st;
}

AttendPlan plan_attend_mfma(const AttendArgs& a, size_t split_ws_bytes) {
  AttendPlan p;
  const int r_heads = a.h_q / a.h_kv;
  const int n_rows = a.n_g * r_heads;
  const int n_rb = ((n_rows + MF_HB - 1) / MF_HB + 1) / 2;
  const int n_wg = n_rb * a.h_kv;
  const int cus = device_cu_count();
  p.mirrored = n_wg <= cus;  // all workgroups resident at once: balance them; otherwise longest first
  p.n_split = 1;
  p.split_rb = 0;
  p.split_tiles = 0;
  p.scratch_bytes = 0;
  const int n_ct = (a.c + MF_BN - 1) / MF_BN;
  const size_t per_row = (size_t)(MF_D + 1) * sizeof(float);  // a partial row and its log-sum-exp
  if (split_ws_bytes > 0 && n_wg < MF_SPLIT_BELOW && n_ct >= 4) {
    // Few rows against a long cache (text prefill, decode, small groups): split the cache of every row block over
    // chunks so that the launch still covers the chip, at most one workgroup per CU, at least two tiles per chunk.
    const size_t per_split = (size_t)a.h_kv * n_rows * per_row;
    long want = cus / n_wg;  // rounded down: all chunks' workgroups resident at once, one round
    want = std::min<long>(want, n_ct / 2);
    want = std::min<long>(want, MF_MAX_SPLIT);
    want = std::min<long>(want, (long)(std::min(split_ws_bytes, MF_SPLIT_ALL_BYTES) / per_split));
    if (want >= 2) {
      p.split_tiles = chunk_tiles(n_ct, (int)want, (a.n_g + MF_BN - 1) / MF_BN);
      p.n_split = (n_ct + p.split_tiles - 1) / p.split_tiles;
      p.split_rb = n_rb;
      p.scratch_bytes = (size_t)p.n_split * per_split;
    }
  } else if (split_ws_bytes > 0 && !p.mirrored && (8 % a.h_kv == 0 || a.h_kv % 8 == 0)) {
    // Several rounds of workgroups, one per CU at a time. The workgroups of a KV head run on the CUs of that head's
    // XCDs (`pool` CUs serve `heads` KV heads); when the last round would fill only part of them, its row blocks (the
    // shortest: earliest tokens, started last) are split into chunks so that the chunks fill the pool evenly: t row
    // blocks in s chunks each take ceil(t s / pool) / s of a round instead of a whole one.
    const int heads = 8 % a.h_kv == 0 ? 1 : a.h_kv / 8;
    const int pool = 8 % a.h_kv == 0 ? cus / a.h_kv : cus / 8;
    const int items = n_rb * heads;
    const int tail = (items % pool) / heads;  // row blocks per KV head in the partial round
    if (pool > 0 && tail > 0) {
      const int part_rows = std::min(n_rows, tail * 2 * MF_HB);
      const int n_gt = (part_rows - 1) / r_heads / MF_BN + 1;  // group tiles the split rows see at most
      double best = 0.9;  // of a round: a split must save at least a tenth of one
      for (int want = 2; want <= MF_TAIL_SPLIT_MAX; ++want) {
        const int st = chunk_tiles(n_ct, want, n_gt);
        const int ns = st > 0 ? (n_ct + st - 1) / st : 0;  // the group tiles of the last chunk can make it fewer than wanted
        if (ns < 2 || st < MF_TAIL_MIN_TILES || (size_t)ns * a.h_kv * part_rows * per_row > split_ws_bytes) continue;
        // a chunk costs its share of the row block plus a prologue (~3 % of a row block of this length and more)
        const double cost = (double)((tail * heads * ns + pool - 1) / pool) / ns + 0.03 * (ns - 1);
        if (cost < best - 1e-9) {
          best = cost;
          p.n_split = ns;
          p.split_tiles = st;
          p.split_rb = tail;
          p.scratch_bytes = (size_t)ns * a.h_kv * part_rows * per_row;
        }
      }
    }
  }
  const int n_items = (n_rb - p.split_rb) + p.split_rb * p.n_split;  // workgroups per KV head
  p.workgroups = n_items * a.h_kv;
  if (8 % a.h_kv == 0) {
    const int per = 8 / a.h_kv;
    p.workgroups = (n_items + per - 1) / per * 8;
  }
  return p;
}

void launch_attend_mfma(const AttendArgs& a_in, void* split_ws, size_t split_ws_bytes, hipStream_t s) {
  static bool attr_set[QP_MAX_DEVICES] = {};
  const int dev = current_device();
  if (dev < 0 || !attr_set[dev]) {
    (void)hipFuncSetAttribute((const void*)attend_mfma_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              MF_STAGES * MF_SLOT);
    (void)hipFuncSetAttribute((const void*)attend_mfma_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              MF_STAGES * MF_SLOT);
    if (dev >= 0) attr_set[dev] = true;
  }
  AttendArgs a = a_in;
  const AttendPlan p = plan_attend_mfma(a, split_ws != nullptr ? split_ws_bytes : 0);
  a.mirrored = p.mirrored;
  a.n_split = p.n_split;
  a.split_tiles = p.split_tiles;
  a.split_rb = p.split_rb;
  a.part_rows = std::min(a.n_g * (a.h_q / a.h_kv), p.split_rb * 2 * MF_HB);
  a.part_o = nullptr;
  a.part_lse = nullptr;
  if (p.n_split > 1) {
    a.part_o = (float*)split_ws;
    a.part_lse = a.part_o + (size_t)p.n_split * a.h_kv * a.part_rows * MF_D;
  }
  if (a.cache_fp8)
    hipLaunchKernelGGL(attend_mfma_kernel<true>, dim3(p.workgroups), dim3(MF_NT), MF_STAGES * MF_SLOT, s, a);
  else
    hipLaunchKernelGGL(attend_mfma_kernel<false>, dim3(p.workgroups), dim3(MF_NT), MF_STAGES * MF_SLOT, s, a);
  if (p.n_split > 1) launch_attend_merge(a, s);
}

void launch_attend_merge(const AttendArgs& a, hipStream_t s) {
  const long total = (long)a.h_kv * a.part_rows;
  // few rows, many chunks (decode, text chunks): a workgroup of 8 wavefronts per row; many rows, few chunks (small
  // video groups): a wavefront per row
  if (total > 1024 && a.n_split <= 16)
    hipLaunchKernelGGL(attend_merge_rows_kernel, dim3((unsigned)((total + MR_WAVES - 1) / MR_WAVES)), dim3(MR_WAVES * 64), 0, s, a);
  else
    hipLaunchKernelGGL(attend_merge_kernel, dim3((unsigned)total), dim3(MG_WAVES * 64), 0, s, a);
}

}  // namespace qp
