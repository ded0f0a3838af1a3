// TopK of Eq. 2 (Sec. 3.2) per KV head, and compaction K~ = K_g[I], V~ = V_g[I] into the cache, in ONE launch.
//
// topk_compact_kernel: grid (slices, KV heads). Every workgroup of a head finds the head's selection threshold
// itself, on order-preserving 32-bit keys held in LDS (the head's scores are a few tens of KB and come from L2, so
// repeating the search costs less than a second launch or a wait between workgroups), and then handles only its own
// slice of the group's tokens: it ranks the slice's survivors, writes their indices and cache positions, and copies
// their K and V rows (16-byte vector loads/stores, d*sizeof/16 lanes per row, all loads of a batch in flight before
// the first store). Copies of early workgroups overlap the searches of later ones.
// When every token is kept (k = N_g) there is nothing to select: append_all_kernel copies the rows in order.
//
// Selection = find the k-th largest key T and how many keys equal to T survive (`need`), then emit.
//   * While loading, the workgroup takes the minimum and maximum key. A round spreads the current key
//     range [lo, lo+span] over up to 2048 buckets of equal power-of-two width (bucket = (key-lo) >> sh),
//     counts keys per bucket with LDS atomics, turns the counts into suffix sums (two buckets per
//     thread, shuffles inside a wavefront, 16 wavefront totals through LDS) and picks the bucket in
//     which the k-th largest key falls; the range shrinks to that bucket. Because the buckets follow the
//     data's own range, real scores (which share sign and exponent) spread over them and the atomics
//     rarely collide; one ballot per batch folds a digit shared by many lanes into a single atomic, so
//     that a constant score vector does not serialise either.
//   * As soon as the bucket holds at most 256 keys they are copied to a list and ranked directly
//     (every candidate counts the candidates above and equal to it). Otherwise another round runs on the
//     bucket; a bucket of width one is exact. The width shrinks by 2^11 per round: at most 3 rounds.
//   * Emit: a token survives iff key > T, or key == T and fewer than `need` equal keys precede it: ties go to
//     the lower index and the kept list comes out in ascending token order. The workgroup counts the
//     (greater, equal) keys before its slice, which fixes where the slice's survivors start; inside the slice
//     wavefront w owns a contiguous run of tokens and walks it 64 at a time, ballots give every survivor its rank
//     inside the batch, running counts its slot.
#include "fp8_e4m3.h"
#include "qp_internal.h"

namespace qp {

constexpr int TOPK_THREADS = 1024;
constexpr int TOPK_WAVES = TOPK_THREADS / 64;
constexpr int SEL_BITS = 11;
constexpr int SEL_NB = 1 << SEL_BITS;  // buckets per round, two per thread
constexpr int SEL_LIST = 256;          // a bucket of at most this many keys is ranked directly
constexpr int SEL_UNROLL = 2;          // independent LDS reads per thread and loop trip
constexpr int LOAD_UNROLL = 8;         // score loads per thread in flight while the keys are brought in
constexpr int SEL_MAX_ROUNDS = 4;      // 3 suffice for 32-bit keys; the bound makes termination explicit
constexpr int GATHER_UNROLL = 4;       // rows per lane group in flight in the copy
constexpr int SLICE_MAX = 4096;        // tokens per slice at most (their survivors' indices sit in LDS)
constexpr int SLICE_WANT_KEEP = 128;   // survivors per slice aimed for
constexpr int SLICES_MAX = 16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
static_assert(SEL_NB == 2 * TOPK_THREADS, "two buckets per thread");

__device__ __forceinline__ uint32_t order_key(float s) {
  s += 0.f;  // -0.0 -> +0.0 so that the two zeros tie
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // ascending in s
}

// 8 bf16 values (16 bytes) as 8 E4M3 codes (the 8-bit cache's rows)
__device__ __forceinline__ uint2 pack8_e4m3(const u32x4& b) {
  uint2 r;
  r.x = bf16_to_e4m3(b.x & 0xffffu) | (bf16_to_e4m3(b.x >> 16) << 8) | (bf16_to_e4m3(b.y & 0xffffu) << 16) |
        (bf16_to_e4m3(b.y >> 16) << 24);
  r.y = bf16_to_e4m3(b.z & 0xffffu) | (bf16_to_e4m3(b.z >> 16) << 8) | (bf16_to_e4m3(b.w & 0xffffu) << 16) |
        (bf16_to_e4m3(b.w >> 16) << 24);
  return r;
}

// keep == n_g (retention 1, and the single tokens and text chunks that follow the video, Sec. 2.1): every token
// survives whatever its score, so the selection is the identity and the compaction a plain append. One lane per 16
// bytes of a row; grid (row runs, KV heads).
constexpr int APPEND_THREADS = 256;
template <typename T, int D>
__global__ __launch_bounds__(APPEND_THREADS) void append_all_kernel(TopkArgs a, int32_t* __restrict__ kept_out) {
  constexpr int PER = Elem<T>::kPer16B;
  constexpr int LPR = D / PER;  // lanes per row
  const int h = blockIdx.y;
  const int idx = blockIdx.x * APPEND_THREADS + threadIdx.x;
  const int j = idx / LPR, sub = idx - j * LPR;
  if (j >= a.n_g) return;
  const size_t src = ((size_t)j * a.h_kv + h) * D + sub * PER;
  const u32x4 kk = *(const u32x4*)((const T*)a.k + src), vv = *(const u32x4*)((const T*)a.v + src);
  const size_t row = (size_t)h * a.cap + a.len + j;
  if (sizeof(T) == 2 && a.cache_fp8) {
    *(uint2*)((unsigned char*)a.ck + row * D + sub * PER) = pack8_e4m3(kk);
    *(uint2*)((unsigned char*)a.cv + row * D + sub * PER) = pack8_e4m3(vv);
  } else {
    *(u32x4*)((T*)a.ck + row * D + sub * PER) = kk;
    *(u32x4*)((T*)a.cv + row * D + sub * PER) = vv;
  }
  if (sub == 0) {
    a.pos[row] = a.base + j;
    if (kept_out != nullptr) kept_out[(size_t)h * a.keep + j] = j;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(TOPK_THREADS) void topk_compact_kernel(TopkArgs a, int32_t* __restrict__ kept_out, int slice_tokens) {
  extern __shared__ uint32_t keys[];  // [n_g] keys, then [slice_tokens] kept token indices of this slice
  __shared__ __attribute__((aligned(8))) uint32_t hist[SEL_NB];
  __shared__ uint32_t list[SEL_LIST];
  __shared__ uint32_t wave_a[TOPK_WAVES], wave_b[TOPK_WAVES], wave_min[TOPK_WAVES], wave_max[TOPK_WAVES];
  __shared__ uint32_t sel_bucket, sel_need, sel_count, sel_key, list_n;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int h = blockIdx.y, n = a.n_g;
  uint32_t* sl_idx = keys + n;
  const float* s = a.scores + (size_t)h * n;
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  for (int j0 = tid; j0 < n; j0 += LOAD_UNROLL * TOPK_THREADS) {
    float f[LOAD_UNROLL];
#pragma unroll
    for (int u = 0; u < LOAD_UNROLL; ++u) f[u] = j0 + u * TOPK_THREADS < n ? s[j0 + u * TOPK_THREADS] : 0.f;
#pragma unroll
    for (int u = 0; u < LOAD_UNROLL; ++u)
      if (j0 + u * TOPK_THREADS < n) {
        const uint32_t key = order_key(f[u]);
        keys[j0 + u * TOPK_THREADS] = key;
        kmin = min(kmin, key);
        kmax = max(kmax, key);
      }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, 64));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, 64));
  }
  if (lane == 0) {
    wave_min[wave] = kmin;
    wave_max[wave] = kmax;
  }
  hist[2 * tid] = 0;
  hist[2 * tid + 1] = 0;
  if (tid == 0) list_n = 0;
  __syncthreads();
  uint32_t lo = 0xffffffffu, hi = 0u;
#pragma unroll
  for (int w = 0; w < TOPK_WAVES; ++w) {  // wavefronts without keys hold the identities
    lo = min(lo, wave_min[w]);
    hi = max(hi, wave_max[w]);
  }

  const int n_round = (n + TOPK_THREADS - 1) / TOPK_THREADS * TOPK_THREADS;  // whole wavefronts take part
  uint32_t span = hi - lo;          // keys still in play: lo <= key <= lo + span
  uint32_t need = (uint32_t)a.keep; // rank of T among them, counted from the largest
  uint32_t thr = lo;
  for (int round = 0; round < SEL_MAX_ROUNDS; ++round) {
    const int bits = span ? 32 - __builtin_clz(span) : 0;
    const int sh = bits > SEL_BITS ? bits - SEL_BITS : 0;
    for (int j0 = tid; j0 < n_round; j0 += SEL_UNROLL * TOPK_THREADS) {
      uint32_t kk[SEL_UNROLL];
#pragma unroll
      for (int u = 0; u < SEL_UNROLL; ++u) kk[u] = j0 + u * TOPK_THREADS < n ? keys[j0 + u * TOPK_THREADS] : 0u;
#pragma unroll
      for (int u = 0; u < SEL_UNROLL; ++u) {
        const int j = j0 + u * TOPK_THREADS;  // j >= n_round only when j >= n: such a batch has no active lane
        const uint32_t off = kk[u] - lo;
        bool act = j < n && off <= span;  // a key below lo wraps to a large offset
        const uint32_t bin = off >> sh;
        const unsigned long long am = __ballot(act);
        if (am != 0) {  // fold the first active lane's bucket when many lanes share it
          const int leader = __ffsll((long long)am) - 1;
          const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
          const bool mine = act && bin == b0;
          const unsigned long long same = __ballot(mine);
          if (__popcll(same) >= 8) {
            if (lane == leader) atomicAdd(&hist[b0], (uint32_t)__popcll(same));
            if (mine) act = false;
          }
        }
        if (act) atomicAdd(&hist[bin], 1u);
      }
    }
    __syncthreads();
    // suffix sums over the buckets: this thread owns buckets 2 tid and 2 tid + 1 (and clears them for a next round)
    const uint2 hb = *(const uint2*)&hist[2 * tid];
    *(uint2*)&hist[2 * tid] = make_uint2(0u, 0u);
    const uint32_t own = hb.x + hb.y;
    uint32_t suf = own;  // inclusive suffix over the wavefront's lanes
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t t = __shfl_down(suf, o, 64);
      if (lane + o < 64) suf += t;
    }
    if (lane == 0) wave_a[wave] = suf;
    __syncthreads();
    uint32_t above = suf - own;  // keys in buckets above 2 tid + 1
#pragma unroll
    for (int w = 1; w < TOPK_WAVES; ++w) above += w > wave ? wave_a[w] : 0u;
    const uint32_t suf1 = above + hb.y, suf0 = suf1 + hb.x;
    if (suf1 >= need && above < need) {  // exactly one (thread, bucket) holds the crossing
      sel_bucket = 2 * tid + 1;
      sel_need = need - above;
      sel_count = hb.y;
    } else if (suf0 >= need && suf1 < need) {
      sel_bucket = 2 * tid;
      sel_need = need - suf1;
      sel_count = hb.x;
    }
    __syncthreads();
    const uint32_t first = sel_bucket << sh;  // offset of the chosen bucket's first key
    need = sel_need;
    const uint32_t count = sel_count;
    lo += first;
    span = min(span - first, (sh ? (1u << sh) : 1u) - 1u);
    thr = lo;
    if (sh == 0) break;  // buckets were single keys: T = lo, `need` of its copies survive
    if (count <= SEL_LIST) {
      // rank the bucket's keys directly
      for (int j = tid; j < n; j += TOPK_THREADS) {
        const uint32_t key = keys[j];
        if (key - lo <= span) {
          const uint32_t p = atomicAdd(&list_n, 1u);
          if (p < (uint32_t)SEL_LIST) list[p] = key;  // always true: the bucket holds `count` keys
        }
      }
      __syncthreads();
      if (tid < (int)count) {
        const uint32_t x = list[tid];
        uint32_t g = 0, e = 0;
        for (uint32_t m = 0; m < count; ++m) {
          const uint32_t y = list[m];
          g += y > x;
          e += y == x;
        }
        if (g < need && need <= g + e) {  // equal candidates write the same values
          sel_key = x;
          sel_need = need - g;
        }
      }
      __syncthreads();
      thr = sel_key;
      need = sel_need;
      break;
    }
  }
  // thr: the k-th largest key; need: how many keys equal to it survive (>= 1)

  // this workgroup's slice of the tokens, and the (greater, equal) keys before it
  const int s_begin = min((int)blockIdx.x * slice_tokens, n), s_end = min(s_begin + slice_tokens, n);
  uint32_t gt_c = 0, eq_c = 0;
  for (int j = tid; j < s_begin; j += TOPK_THREADS) {
    const uint32_t key = keys[j];
    gt_c += key > thr;
    eq_c += key == thr;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    gt_c += (uint32_t)__shfl_xor((int)gt_c, o, 64);
    eq_c += (uint32_t)__shfl_xor((int)eq_c, o, 64);
  }
  // emit, wavefront by wavefront over contiguous runs of the slice's tokens
  const int run = ((s_end - s_begin + TOPK_WAVES - 1) / TOPK_WAVES + 63) / 64 * 64;
  const int j_begin = min(s_begin + wave * run, s_end), j_end = min(j_begin + run, s_end);
  uint32_t gt_w = 0, eq_w = 0;
  for (int j0 = j_begin; j0 < j_end; j0 += 64 * SEL_UNROLL) {
    uint32_t kk[SEL_UNROLL];
#pragma unroll
    for (int u = 0; u < SEL_UNROLL; ++u) kk[u] = j0 + 64 * u + lane < j_end ? keys[j0 + 64 * u + lane] : 0u;
#pragma unroll
    for (int u = 0; u < SEL_UNROLL; ++u) {
      const bool in = j0 + 64 * u + lane < j_end;
      gt_w += (uint32_t)__popcll(__ballot(in && kk[u] > thr));
      eq_w += (uint32_t)__popcll(__ballot(in && kk[u] == thr));
    }
  }
  __syncthreads();  // wave_a / wave_b of the threshold search are free again
  if (lane == 0) {
    wave_a[wave] = gt_w;
    wave_b[wave] = eq_w;
    wave_min[wave] = gt_c;  // the counts before the slice, per wavefront
    wave_max[wave] = eq_c;
  }
  __syncthreads();
  uint32_t gt_before = 0, eq_before = 0, gt_run = 0, eq_run = 0, gt_slice = 0, eq_slice = 0;
#pragma unroll
  for (int w = 0; w < TOPK_WAVES; ++w) {
    gt_before += wave_min[w];
    eq_before += wave_max[w];
    gt_run += w < wave ? wave_a[w] : 0u;
    eq_run += w < wave ? wave_b[w] : 0u;
    gt_slice += wave_a[w];
    eq_slice += wave_b[w];
  }
  const uint32_t out_base = gt_before + min(eq_before, need);  // slot of the slice's first survivor
  const uint32_t n_slice = gt_slice + (min(eq_before + eq_slice, need) - min(eq_before, need));
  eq_run += eq_before;
  uint32_t out_run = gt_before + gt_run + min(eq_run, need);
  int32_t* pos = a.pos + (size_t)h * a.cap + a.len;
  const unsigned long long below = (1ull << lane) - 1ull;  // lanes before this one
  for (int j0 = j_begin; j0 < j_end; j0 += 64 * SEL_UNROLL) {
    uint32_t kk[SEL_UNROLL];
#pragma unroll
    for (int u = 0; u < SEL_UNROLL; ++u) kk[u] = j0 + 64 * u + lane < j_end ? keys[j0 + 64 * u + lane] : 0u;
#pragma unroll
    for (int u = 0; u < SEL_UNROLL; ++u) {
      const int j = j0 + 64 * u + lane;
      const bool is_eq = j < j_end && kk[u] == thr;
      const unsigned long long be = __ballot(is_eq);
      const bool keep_it = (j < j_end && kk[u] > thr) || (is_eq && eq_run + (uint32_t)__popcll(be & below) < need);
      const unsigned long long bs = __ballot(keep_it);
      const uint32_t slot = out_run + (uint32_t)__popcll(bs & below);
      // out_base <= slot < out_base + n_slice <= keep always holds; the checks keep the stores in bounds
      if (keep_it && slot < (uint32_t)a.keep && slot - out_base < (uint32_t)slice_tokens) {
        sl_idx[slot - out_base] = (uint32_t)j;
        if (kept_out != nullptr) kept_out[(size_t)h * a.keep + slot] = j;
        pos[slot] = a.base + j;
      }
      out_run += (uint32_t)__popcll(bs);
      eq_run += (uint32_t)__popcll(be);
    }
  }
  __syncthreads();

  // copy the slice's survivors: row r of the slice goes to cache row len + out_base + r
  constexpr int PER = Elem<T>::kPer16B;
  constexpr int LPR = D / PER;  // lanes per row
  constexpr int ROWS_PER_ITER = TOPK_THREADS / LPR;
  const int sub = tid % LPR;
  const int n_copy = (int)min(n_slice, (uint32_t)min(slice_tokens, a.keep - (int)min(out_base, (uint32_t)a.keep)));
  const T* gk = (const T*)a.k;
  const T* gv = (const T*)a.v;
  T* ck = (T*)a.ck + ((size_t)h * a.cap + a.len + out_base) * D;
  T* cv = (T*)a.cv + ((size_t)h * a.cap + a.len + out_base) * D;
  const bool to_fp8 = sizeof(T) == 2 && a.cache_fp8;  // 8-bit cache rows: one byte per element, 8 bytes per lane
  unsigned char* ck8 = (unsigned char*)a.ck + ((size_t)h * a.cap + a.len + out_base) * D;
  unsigned char* cv8 = (unsigned char*)a.cv + ((size_t)h * a.cap + a.len + out_base) * D;
  for (int r0 = tid / LPR; r0 < n_copy; r0 += ROWS_PER_ITER * GATHER_UNROLL) {
    u32x4 kk[GATHER_UNROLL], vv[GATHER_UNROLL];
#pragma unroll
    for (int u = 0; u < GATHER_UNROLL; ++u) {
      const int r = r0 + u * ROWS_PER_ITER;
      if (r < n_copy) {
        const size_t src = ((size_t)sl_idx[r] * a.h_kv + h) * D + sub * PER;
        kk[u] = *(const u32x4*)(gk + src);
        vv[u] = *(const u32x4*)(gv + src);
      }
    }
#pragma unroll
    for (int u = 0; u < GATHER_UNROLL; ++u) {
      const int r = r0 + u * ROWS_PER_ITER;
      if (r < n_copy) {
        const size_t dst = (size_t)r * D + sub * PER;
        if (to_fp8) {
          *(uint2*)(ck8 + dst) = pack8_e4m3(kk[u]);  // dst counts elements = bytes here
          *(uint2*)(cv8 + dst) = pack8_e4m3(vv[u]);
        } else {
          *(u32x4*)(ck + dst) = kk[u];
          *(u32x4*)(cv + dst) = vv[u];
        }
      }
    }
  }
}

size_t topk_workspace_bytes(int h_kv, int keep) { return ((size_t)h_kv * keep * sizeof(int32_t) + 255) / 256 * 256; }

// Tokens per slice: about SLICE_WANT_KEEP survivors each, at most SLICES_MAX slices and about one workgroup per
// compute unit over all heads, at most SLICE_MAX tokens, whole batches of 64.
static int slice_tokens_for(int n_g, int keep, int h_kv) {
  int slices = (keep + SLICE_WANT_KEEP - 1) / SLICE_WANT_KEEP;
  if (slices > SLICES_MAX) slices = SLICES_MAX;
  // every workgroup repeats the head's threshold search: with many heads there are enough workgroups without
  // slicing, and more than one per compute unit only multiplies that search
  const int per_head = device_cu_count() / h_kv;
  if (slices > per_head) slices = per_head;
  const int at_least = (n_g + SLICE_MAX - 1) / SLICE_MAX;
  if (slices < at_least) slices = at_least;
  if (slices < 1) slices = 1;
  return ((n_g + slices - 1) / slices + 63) / 64 * 64;  // <= SLICE_MAX: SLICE_MAX is a multiple of 64
}

template <typename T, int D>
static hipError_t launch_fused(const TopkArgs& a, int32_t* kept_out, hipStream_t s) {
  if (a.keep == a.n_g) {  // nothing to select
    constexpr int LPR = D / Elem<T>::kPer16B;
    hipLaunchKernelGGL((append_all_kernel<T, D>), dim3((a.n_g * LPR + APPEND_THREADS - 1) / APPEND_THREADS, a.h_kv),
                       dim3(APPEND_THREADS), 0, s, a, kept_out);
    return hipSuccess;
  }
  const int slice_tokens = slice_tokens_for(a.n_g, a.keep, a.h_kv);
  const int slices = (a.n_g + slice_tokens - 1) / slice_tokens;
  const size_t lds_bytes = ((size_t)a.n_g + slice_tokens) * sizeof(uint32_t);
  static bool attr_set[QP_MAX_DEVICES] = {};
  const int dev = current_device();
  if (dev < 0 || !attr_set[dev]) {
    hipError_t e = hipFuncSetAttribute((const void*)topk_compact_kernel<T, D>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (QP_MAX_GROUP_TOKENS + SLICE_MAX) * (int)sizeof(uint32_t));
    if (e != hipSuccess) return e;
    if (dev >= 0) attr_set[dev] = true;
  }
  hipLaunchKernelGGL((topk_compact_kernel<T, D>), dim3(slices, a.h_kv), dim3(TOPK_THREADS), lds_bytes, s, a, kept_out,
                     slice_tokens);
  return hipSuccess;
}

// kept_out: [h_kv][keep] int32 for the kept indices, or nullptr if the caller does not want them
hipError_t launch_topk_compact(const TopkArgs& a, int dtype, int32_t* kept_out, hipStream_t s) {
  if (dtype == QP_F32) return a.d == 64 ? launch_fused<float, 64>(a, kept_out, s) : launch_fused<float, 128>(a, kept_out, s);
  return a.d == 64 ? launch_fused<bf16_t, 64>(a, kept_out, s) : launch_fused<bf16_t, 128>(a, kept_out, s);
}

}  // namespace qp
