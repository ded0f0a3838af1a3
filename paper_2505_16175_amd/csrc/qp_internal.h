// Internal declarations shared by the translation units of libqp_hip.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qp.h"

namespace qp {

// bf16 is handled as raw 16-bit patterns: widening is a shift, narrowing is round-to-nearest-even.
typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
__device__ __forceinline__ bf16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int kPer16B = 4;
};
template <>
struct Elem<bf16_t> {
  static constexpr int kPer16B = 8;
};

// Widen one 16-byte chunk (uint4) of T into kPer16B floats.
template <typename T>
__device__ __forceinline__ void widen16(const uint4& raw, float* out);
template <>
__device__ __forceinline__ void widen16<float>(const uint4& raw, float* out) {
  out[0] = __uint_as_float(raw.x);
  out[1] = __uint_as_float(raw.y);
  out[2] = __uint_as_float(raw.z);
  out[3] = __uint_as_float(raw.w);
}
template <>
__device__ __forceinline__ void widen16<bf16_t>(const uint4& raw, float* out) {
  out[0] = bf16lo_to_f32(raw.x);
  out[1] = bf16hi_to_f32(raw.x);
  out[2] = bf16lo_to_f32(raw.y);
  out[3] = bf16hi_to_f32(raw.y);
  out[4] = bf16lo_to_f32(raw.z);
  out[5] = bf16hi_to_f32(raw.z);
  out[6] = bf16lo_to_f32(raw.w);
  out[7] = bf16hi_to_f32(raw.w);
}

template <typename T>
__device__ __forceinline__ void store_elem(T* p, float v);
template <>
__device__ __forceinline__ void store_elem<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_elem<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16_rne(v); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// max / sum of x over the lane pair (l, l ^ 32), i.e. over the two halves of the wavefront, by v_permlane32_swap:
// afterwards one register holds the lower half's values in both halves and the other the upper half's. A vector-ALU
// operation, where a shuffle through the LDS crossbar (ds_bpermute) would also make the wavefront wait for all of
// its pending LDS reads.
__device__ __forceinline__ float max_halves(float x) {
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}
__device__ __forceinline__ float sum_halves(float x) {
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}

// 64 lanes x 16 bytes global -> LDS without passing through registers: lane L's chunk lands at
// lds_dst + 16 L (lds_dst is wave-uniform). Written as inline assembly so that the compiler does not
// treat it as an LDS store it must drain (vmcnt(0)) before every later LDS read; the kernel waits for
// these loads itself (s_waitcnt vmcnt) before the barrier that publishes a tile. m0 is on the clobber list so that
// the compiler orders its own uses of m0 around the statement (it warns that m0 is reserved: nothing is to be
// preserved here, the statement sets m0 itself each time).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma16(const unsigned char* base, unsigned byte_off, unsigned char* lds_dst) {
  const unsigned lds_addr =
      __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds_dst);
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(byte_off), "s"(base), "s"(lds_addr)
      : "memory", "m0");
}
#pragma clang diagnostic pop

// Arguments common to the attention kernels. All pointers are device pointers.
struct AttendArgs {
  const void* q;      // [n_g][h_q][d]
  const void* k;      // [n_g][h_kv][d]
  const void* v;      // [n_g][h_kv][d]
  const void* ck;     // [h_kv][cap][d] or nullptr when c == 0
  const void* cv;
  void* out;          // [n_g][h_q][d]
  float* lse;         // [h_q][n_g] or nullptr
  int n_g, h_q, h_kv, d, c, cap;
  int cache_fp8;      // 1: ck / cv hold one E4M3 byte per element (MFMA and decode kernels)
  float scale_log2;   // softmax scale * log2(e)
  // Key split of the MFMA kernel: the cache tiles of a split row block are dealt to n_split chunks of split_tiles
  // tiles, the last chunk also takes the group's own tiles; every chunk leaves a normalised partial output and its
  // log2-sum-exp, merged by a second launch. n_split == 1: no split, nothing below is used. The split_rb row blocks
  // with the EARLIEST tokens are split (rows 0 .. part_rows-1 of every KV head), the others are served by one
  // workgroup each: all of them for few rows against a long cache, the last partial round of workgroups otherwise.
  int n_split, split_tiles;
  int split_rb;       // row blocks (256 rows) that are split, counted from the group's first token
  int part_rows;      // rows per KV head that have partials: min(n_g * R, 256 * split_rb)
  int mirrored;       // MFMA kernel's row mapping: 1 = mirrored half blocks (balanced), 0 = consecutive, longest first
  float* part_o;      // [n_split][h_kv * part_rows][d] f32
  float* part_lse;    // [n_split][h_kv * part_rows]    f32, log2 units
};

// Launchers (defined next to their kernels). They only enqueue; hipGetLastError is checked by the caller.
void launch_attend_scalar(const AttendArgs& a, int dtype, hipStream_t s);
bool attend_mfma_supported(const AttendArgs& a, int dtype);
// How launch_attend_mfma lays a call out: grid (one-dimensional), key split, row mapping, scratch it takes.
struct AttendPlan {
  int workgroups;       // grid size: whole row blocks and chunks of all KV heads, plus the padding of the XCD mapping
  int n_split;          // key chunks of a split row block (1 = no split)
  int split_rb;         // row blocks per KV head that are split (all of them, or the launch's last partial round)
  int split_tiles;      // cache tiles per chunk
  int mirrored;         // row mapping, see AttendArgs
  size_t scratch_bytes; // bytes of the split scratch used (0 without split)
};
// split_ws_bytes: scratch the caller can offer for the key split (0: never split). Host arithmetic only.
AttendPlan plan_attend_mfma(const AttendArgs& a, size_t split_ws_bytes);
// split_ws / split_ws_bytes: optional scratch (256-byte aligned) for the key split; without it the kernel never splits
void launch_attend_mfma(const AttendArgs& a, void* split_ws, size_t split_ws_bytes, hipStream_t s);

void launch_attend_merge(const AttendArgs& a, hipStream_t s);  // merges a.n_split partials (a.part_o, a.part_lse)
// Decode-shaped launches (at most 32 stacked rows per KV head): every wavefront streams its own key blocks.
bool attend_decode_applies(const AttendArgs& a, int dtype);
AttendPlan plan_attend_decode(const AttendArgs& a, size_t split_ws_bytes);  // n_split = workgroups per KV head
void launch_attend_decode(const AttendArgs& a, void* split_ws, size_t split_ws_bytes, hipStream_t s);

// Per-device host state (kernel attributes, library streams, CU count) is kept in arrays of this many slots.
constexpr int QP_MAX_DEVICES = 64;
int current_device();   // index of the current HIP device, -1 if there is none or it does not fit the arrays
int device_cu_count();  // compute units of the current device; 256 (MI355X) if it cannot be asked
void note_hip_error(int e);  // what qp_last_hip_error() reports on this thread
// The device's library-owned side stream, ordered after `main`'s work so far (nullptr if there is none); a non-null
// return holds the library's enqueue mutex until side_join(main), which makes `main` wait for the side stream.
hipStream_t side_fork(hipStream_t main);
void side_join(hipStream_t main);

void launch_score_norm(const void* x, int dtype, int n_g, int h_kv, int d, float sign, float* scores, hipStream_t s);

struct WindowArgs {
  const void* k;      // [n_g][h_kv][d]
  const void* q_win;  // [w][h_q][d]
  float* scores;      // [h_kv][n_g]
  void* workspace;
  int n_g, h_q, h_kv, d, w;
  float scale_log2;
};
size_t window_workspace_bytes(int h_q, int h_kv, int n_g, int w);
size_t window_logit_workspace_bytes(int h_kv, int d);  // the summed window rows, [h_kv][d] f32
void launch_score_window_logit(const WindowArgs& a, int dtype, float scale, hipStream_t s);
void launch_share_heads(float* scores, int h_kv, int n_g, hipStream_t s);
void launch_score_window(const WindowArgs& a, int dtype, hipStream_t s);
bool window_mfma_supported(int dtype, int h_q, int h_kv, int d, int w);
size_t window_mfma_workspace_bytes(int h_q, int h_kv, int n_g, int w);
void launch_score_window_mfma(const WindowArgs& a, hipStream_t s);

struct TopkArgs {
  const float* scores;  // [h_kv][n_g]
  const void* k;        // [n_g][h_kv][d]
  const void* v;
  void* ck;             // [h_kv][cap][d]
  void* cv;
  int32_t* pos;         // [h_kv][cap]
  int n_g, h_kv, d, keep, base, cap, len;
  int cache_fp8;        // 1: ck / cv take one E4M3 byte per element (bf16 inputs only)
};
size_t topk_workspace_bytes(int h_kv, int keep);
hipError_t launch_topk_compact(const TopkArgs& a, int dtype, int32_t* kept_ws, hipStream_t s);

// ---- decoder layer around the path: projections with fused elementwise steps, RMSNorm, rotary table ----
enum GemmMode { GEMM_PLAIN = 0, GEMM_QKV_ROPE = 1, GEMM_SWIGLU = 2 };
struct GemmArgs {
  const void* x;         // [m][k] bf16 activations
  const void* w;         // [n][k] bf16 weights ([out][in]); SWIGLU: n = 2 d_ff, gate rows then up rows
  const void* bias;      // [n] bf16 or nullptr (PLAIN); required for QKV_ROPE
  const void* residual;  // [m][n] bf16 or nullptr (PLAIN)
  void* out;             // PLAIN: [m][n]; SWIGLU: [m][n / 2]
  void* q;               // QKV_ROPE: [m][h_q][128]
  void* k_out;           //           [m][h_kv][128]
  void* v_out;           //           [m][h_kv][128]
  const float* cos_sin;  // QKV_ROPE: [m][64][2] f32, (cos, sin) of each token's 64 rotation angles
  int m, n, k;
  int h_q, h_kv;
  int tiles_m, tiles_n, m_block, n_quads;  // filled by the launcher (tile counts and the XCD block mapping)
  int split_k, steps_per_split;            // filled by the launcher: k chunks (1 = none) and 64-wide k-steps per chunk
  float* partial;                          // [split_k][m][n] f32 partial sums when split_k > 1
};
bool gemm_supported(const GemmArgs& a, int mode);
// scratch: optional (256-byte aligned) room for the partial sums of a split contraction; without it nothing is split
hipError_t launch_gemm_bf16(const GemmArgs& a, int mode, void* scratch, size_t scratch_bytes, hipStream_t s);
struct GemmSplit {
  int split_k, steps_per_split;
  size_t scratch_bytes;
};
GemmSplit gemm_plan_split(const GemmArgs& a, int mode, size_t scratch_bytes);  // host arithmetic only
// Calls of at most 2 tokens stream the weights once through a kernel of their own (one launch, no partial sums).
bool gemv_applies(const GemmArgs& a);
bool gemm_uses_gemv(const GemmArgs& a);   // gemv_applies and no tiling is forced
hipError_t launch_gemv_bf16(const GemmArgs& a, int mode, hipStream_t s);
int gemm_tile_rows(const GemmArgs& a);    // token rows per workgroup tile the launcher would use: 128 or 256
void gemm_force_tile_rows(int rows);      // 0 = choose per launch (default), 128 or 256
void launch_rms_norm(const void* x, const void* w, void* out, int n_tokens, int d_model, float eps, hipStream_t s);
void launch_rope_table(const int32_t* pos, long axis_stride, int n_tokens, float theta, int s0, int s1, float* cos_sin,
                       hipStream_t s);

}  // namespace qp
