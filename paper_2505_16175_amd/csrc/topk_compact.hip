// TopK of Eq. 2 (Sec. 3.2) per KV head, and compaction K~ = K_g[I], V~ = V_g[I] into the cache.
//
// One launch. The grid is (n_split, H_kv); every workgroup of a KV head runs the same
// selection (it is a few microseconds on <= 128 KB of LDS-resident scores, cheaper than a
// second launch) and then copies its own slice of the surviving rows.
//
// Selection = exact radix select on order-preserving 32-bit keys held in LDS:
//   4 passes of 8 bits from the top: histogram (LDS atomics) of the digit among the keys that
//   match the prefix found so far, suffix-sum over the 256 bins (one wavefront, shuffles), pick
//   the bin in which the k-th largest key falls. After 4 passes the prefix is the exact k-th largest key T and
//   `need` is how many keys equal to T survive. Ties go to the lower token index because
//   the compaction below walks tokens in index order: a token survives iff key > T, or
//   key == T and fewer than `need` equal keys precede it. A block-wide exclusive scan of the
//   per-thread (greater, equal) counts over contiguous token chunks gives each survivor its
//   output slot, so the kept list is in ascending token order.
// Copy = 16-byte vector loads/stores, one row (d elements) per d*sizeof/16 lanes.
#include "qp_internal.h"

namespace qp {

constexpr int TOPK_THREADS = 1024;

__device__ __forceinline__ uint32_t order_key(float s) {
  s += 0.f;  // -0.0 -> +0.0 so that the two zeros tie
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // ascending in s
}

template <typename T, int D>
__global__ __launch_bounds__(TOPK_THREADS) void topk_compact_kernel(TopkArgs a) {
  extern __shared__ uint32_t lds[];
  uint32_t* keys = lds;                 // [n_g]
  uint32_t* kept = lds + a.n_g;         // [rows_per]: this workgroup's slice of the kept list
  __shared__ __attribute__((aligned(16))) uint32_t hist[256];
  __shared__ uint32_t wave_gt[TOPK_THREADS / 64], wave_eq[TOPK_THREADS / 64];
  __shared__ uint32_t sel_prefix, sel_need;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int h = blockIdx.y;
  const float* s = a.scores + (size_t)h * a.n_g;
  for (int j = tid; j < a.n_g; j += TOPK_THREADS) keys[j] = order_key(s[j]);
  if (tid == 0) {
    sel_prefix = 0;
    sel_need = (uint32_t)a.keep;
  }
  __syncthreads();

  uint32_t mask = 0;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = sel_prefix;
    for (int j = tid; j < a.n_g; j += TOPK_THREADS) {
      const uint32_t key = keys[j];
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
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
  const uint32_t thr = sel_prefix;   // the k-th largest key
  const uint32_t need = sel_need;    // how many keys equal to it survive (>= 1)

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
  // this workgroup keeps the slice [r0, r1) of the survivors' list
  const int n_split = gridDim.x;
  const int rows_per = (a.keep + n_split - 1) / n_split;
  const int r0 = blockIdx.x * rows_per, r1 = min(r0 + rows_per, a.keep);
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
    if (slot >= r0 && slot < r1) kept[slot - r0] = (uint32_t)j;
  }
  __syncthreads();

  if (a.kept != nullptr)
    for (int r = r0 + tid; r < r1; r += TOPK_THREADS) a.kept[(size_t)h * a.keep + r] = (int32_t)kept[r - r0];
  for (int r = r0 + tid; r < r1; r += TOPK_THREADS)
    a.pos[(size_t)h * a.cap + a.len + r] = a.base + (int32_t)kept[r - r0];

  constexpr int PER = Elem<T>::kPer16B;
  constexpr int LPR = D / PER;                      // lanes per row
  constexpr int ROWS_PER_ITER = TOPK_THREADS / LPR;
  const int sub = tid % LPR;
  const T* gk = (const T*)a.k;
  const T* gv = (const T*)a.v;
  T* ck = (T*)a.ck + ((size_t)h * a.cap + a.len) * D;
  T* cv = (T*)a.cv + ((size_t)h * a.cap + a.len) * D;
  for (int r = r0 + tid / LPR; r < r1; r += ROWS_PER_ITER) {
    const size_t src = ((size_t)kept[r - r0] * a.h_kv + h) * D + sub * PER;
    const size_t dst = (size_t)r * D + sub * PER;
    const uint4 kk = *(const uint4*)(gk + src);
    const uint4 vv = *(const uint4*)(gv + src);
    *(uint4*)(ck + dst) = kk;
    *(uint4*)(cv + dst) = vv;
  }
}

template <typename T, int D>
static hipError_t launch_t(const TopkArgs& a, hipStream_t s) {
  // >= 64 rows (32 KB of K+V at d=128 bf16) per workgroup, and about two workgroups per CU over all heads
  int n_split = (a.keep + 63) / 64;
  const int cap = 512 / a.h_kv > 1 ? 512 / a.h_kv : 1;
  if (n_split > cap) n_split = cap;
  if (n_split > 32) n_split = 32;
  if (n_split < 1) n_split = 1;
  const int rows_per = (a.keep + n_split - 1) / n_split;
  const size_t lds_bytes = ((size_t)a.n_g + rows_per) * sizeof(uint32_t);
  auto kern = topk_compact_kernel<T, D>;
  if (lds_bytes > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3(n_split, a.h_kv), dim3(TOPK_THREADS), lds_bytes, s, a);
  return hipSuccess;
}

hipError_t launch_topk_compact(const TopkArgs& a, int dtype, hipStream_t s) {
  if (dtype == QP_F32) return a.d == 64 ? launch_t<float, 64>(a, s) : launch_t<float, 128>(a, s);
  return a.d == 64 ? launch_t<bf16_t, 64>(a, s) : launch_t<bf16_t, 128>(a, s);
}

}  // namespace qp
