// TopK of Eq. 2 (Sec. 3.2) per KV head, and compaction K~ = K_g[I], V~ = V_g[I] into the cache.
//
// Two launches on the same stream:
//   topk_select_kernel     one workgroup per KV head; exact radix select on order-preserving 32-bit keys
//                          held in LDS; writes the kept indices (ascending) and the cache positions.
//   compact_gather_kernel  pure copy: 16-byte vector loads/stores, one row (d elements) per
//                          d*sizeof/16 lanes, four rows per lane group in flight, 64 rows per workgroup.
//
// Selection: 4 passes of 8 bits from the top. Each pass builds the histogram of the digit among the
// keys that match the prefix found so far (LDS atomics; the two most common digits of every
// wavefront-wide batch are first aggregated with ballots, because real scores share sign and
// exponent, so the first pass would otherwise serialise thousands of atomics on one bin), one
// wavefront turns it into suffix sums with shuffles and picks the bin in which the k-th largest key
// falls. After 4 passes the prefix is the exact k-th largest key T and `need` is how many keys equal
// to T survive. Ties go to the lower token index because the compaction walks tokens in index
// order: a token survives iff key > T, or key == T and fewer than `need` equal keys precede it. A
// block-wide exclusive scan of the per-thread (greater, equal) counts over contiguous token
// chunks gives each survivor its output slot, so the kept list is in ascending token order.
#include "qp_internal.h"

namespace qp {

constexpr int TOPK_THREADS = 1024;
constexpr int GATHER_THREADS = 256;
constexpr int GATHER_UNROLL = 4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t order_key(float s) {
  s += 0.f;  // -0.0 -> +0.0 so that the two zeros tie
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // ascending in s
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_select_kernel(TopkArgs a, int32_t* __restrict__ kept_out) {
  extern __shared__ uint32_t keys[];  // [n_g]
  __shared__ __attribute__((aligned(16))) uint32_t hist[256];
  __shared__ uint32_t wave_gt[TOPK_THREADS / 64], wave_eq[TOPK_THREADS / 64];
  __shared__ uint32_t sel_prefix, sel_need;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int h = blockIdx.x;
  const float* s = a.scores + (size_t)h * a.n_g;
  for (int j = tid; j < a.n_g; j += TOPK_THREADS) keys[j] = order_key(s[j]);
  if (tid == 0) {
    sel_prefix = 0;
    sel_need = (uint32_t)a.keep;
  }
  __syncthreads();

  const int n_round = (a.n_g + TOPK_THREADS - 1) / TOPK_THREADS * TOPK_THREADS;  // whole wavefronts take part
  uint32_t mask = 0;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = sel_prefix;
    for (int j = tid; j < n_round; j += TOPK_THREADS) {
      const uint32_t key = j < a.n_g ? keys[j] : 0u;
      bool act = j < a.n_g && (key & mask) == prefix;
      const uint32_t bin = (key >> shift) & 255u;
      // aggregate the two most common digits of this wavefront's batch, plain atomics for the rest
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const unsigned long long am = __ballot(act);
        if (am == 0) break;
        const int leader = __ffsll((long long)am) - 1;
        const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
        const bool mine = act && bin == b0;
        const unsigned long long same = __ballot(mine);
        if (lane == leader) atomicAdd(&hist[b0], (uint32_t)__popcll(same));
        if (mine) act = false;
      }
      if (act) atomicAdd(&hist[bin], 1u);
    }
    __syncthreads();
    // Wavefront 0 finds the bin of the k-th largest key: lane l owns bins 4l..4l+3; suffix sums (number of
    // matching keys with digit >= b) come from an in-lane sum plus a suffix scan over the lanes.
    if (tid < 64) {
      const uint32_t need = sel_need;
      const uint4 hb = *(const uint4*)&hist[4 * tid];
      const uint32_t s3 = hb.w, s2 = s3 + hb.z, s1 = s2 + hb.y, s0 = s1 + hb.x;
      uint32_t above = s0;  // inclusive suffix over lanes
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_down(above, o, 64);
        if (tid + o < 64) above += t;
      }
      above -= s0;  // keys in bins owned by higher lanes
      const uint32_t suf[5] = {above + s0, above + s1, above + s2, above + s3, above};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (suf[j] >= need && suf[j + 1] < need) {  // true for exactly one (lane, j)
          sel_prefix = prefix | ((uint32_t)(4 * tid + j) << shift);
          sel_need = need - suf[j + 1];
        }
    }
    mask |= 255u << shift;
    __syncthreads();
  }
  const uint32_t thr = sel_prefix;  // the k-th largest key
  const uint32_t need = sel_need;   // how many keys equal to it survive (>= 1)

  // ordered compaction over contiguous chunks of tokens
  const int per = (a.n_g + TOPK_THREADS - 1) / TOPK_THREADS;
  const int j0 = tid * per, j1 = min(j0 + per, a.n_g);
  uint32_t gt = 0, eq = 0;
  for (int j = j0; j < j1; ++j) {
    const uint32_t key = keys[j];
    gt += key > thr;
    eq += key == thr;
  }
  uint32_t gt_inc = gt, eq_inc = eq;  // inclusive scan inside the wave
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t g2 = __shfl_up(gt_inc, o, 64), e2 = __shfl_up(eq_inc, o, 64);
    if (lane >= o) {
      gt_inc += g2;
      eq_inc += e2;
    }
  }
  if (lane == 63) {
    wave_gt[wave] = gt_inc;
    wave_eq[wave] = eq_inc;
  }
  __syncthreads();
  uint32_t gt_before = gt_inc - gt, eq_before = eq_inc - eq;
  for (int w = 0; w < wave; ++w) {
    gt_before += wave_gt[w];
    eq_before += wave_eq[w];
  }
  int32_t* kept = kept_out + (size_t)h * a.keep;
  int32_t* pos = a.pos + (size_t)h * a.cap + a.len;
  for (int j = j0; j < j1; ++j) {
    const uint32_t key = keys[j];
    int slot = -1;
    if (key > thr) {
      slot = (int)(gt_before + min(eq_before, need));
      ++gt_before;
    } else if (key == thr) {
      if (eq_before < need) slot = (int)(gt_before + eq_before);
      ++eq_before;
    }
    if (slot >= 0) {
      kept[slot] = j;
      pos[slot] = a.base + j;
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__(GATHER_THREADS) void compact_gather_kernel(TopkArgs a, const int32_t* __restrict__ kept_in) {
  constexpr int PER = Elem<T>::kPer16B;
  constexpr int LPR = D / PER;  // lanes per row
  constexpr int ROWS_PER_ITER = GATHER_THREADS / LPR;
  const int tid = threadIdx.x, sub = tid % LPR;
  const int h = blockIdx.y;
  const int32_t* kept = kept_in + (size_t)h * a.keep;
  const T* gk = (const T*)a.k;
  const T* gv = (const T*)a.v;
  T* ck = (T*)a.ck + ((size_t)h * a.cap + a.len) * D;
  T* cv = (T*)a.cv + ((size_t)h * a.cap + a.len) * D;
  const int rbase = blockIdx.x * (ROWS_PER_ITER * GATHER_UNROLL) + tid / LPR;
  // four rows per lane group in flight: all loads are issued before the first store
  u32x4 kk[GATHER_UNROLL], vv[GATHER_UNROLL];
#pragma unroll
  for (int u = 0; u < GATHER_UNROLL; ++u) {
    const int r = rbase + u * ROWS_PER_ITER;
    if (r < a.keep) {
      const size_t src = ((size_t)kept[r] * a.h_kv + h) * D + sub * PER;
      kk[u] = *(const u32x4*)(gk + src);
      vv[u] = *(const u32x4*)(gv + src);
    }
  }
#pragma unroll
  for (int u = 0; u < GATHER_UNROLL; ++u) {
    const int r = rbase + u * ROWS_PER_ITER;
    if (r < a.keep) {
      const size_t dst = (size_t)r * D + sub * PER;
      *(u32x4*)(ck + dst) = kk[u];
      *(u32x4*)(cv + dst) = vv[u];
    }
  }
}

size_t topk_workspace_bytes(int h_kv, int keep) { return ((size_t)h_kv * keep * sizeof(int32_t) + 255) / 256 * 256; }

template <typename T, int D>
static void launch_gather(const TopkArgs& a, const int32_t* kept, hipStream_t s) {
  constexpr int ROWS_PER_WG = GATHER_THREADS / (D / Elem<T>::kPer16B) * GATHER_UNROLL;
  hipLaunchKernelGGL((compact_gather_kernel<T, D>), dim3((a.keep + ROWS_PER_WG - 1) / ROWS_PER_WG, a.h_kv),
                     dim3(GATHER_THREADS), 0, s, a, kept);
}

// kept_ws: [h_kv][keep] int32 scratch for the kept indices (the caller's kept buffer or the workspace)
hipError_t launch_topk_compact(const TopkArgs& a, int dtype, int32_t* kept_ws, hipStream_t s) {
  const size_t lds_bytes = (size_t)a.n_g * sizeof(uint32_t);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)topk_select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       QP_MAX_GROUP_TOKENS * (int)sizeof(uint32_t));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(topk_select_kernel, dim3(a.h_kv), dim3(TOPK_THREADS), lds_bytes, s, a, kept_ws);
  if (dtype == QP_F32) {
    if (a.d == 64) launch_gather<float, 64>(a, kept_ws, s);
    else launch_gather<float, 128>(a, kept_ws, s);
  } else {
    if (a.d == 64) launch_gather<bf16_t, 64>(a, kept_ws, s);
    else launch_gather<bf16_t, 128>(a, kept_ws, s);
  }
  return hipSuccess;
}

}  // namespace qp
