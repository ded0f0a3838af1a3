// C-ABI entry points of libqp_hip.so: argument validation, workspace carving, launches,
// and the per-layer group loop of QuickPrefill (Sec. 3.2). Host code only; kernels live in
// the other translation units.
#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "fp8_e4m3.h"
#include "qp_internal.h"

namespace {

thread_local int g_last_hip_error = 0;
std::atomic<int> g_attend_kernel{QP_ATTEND_AUTO};  // read once per call; set by qp_select_attend_kernel from any thread

inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }
inline size_t round256(size_t x) { return (x + 255) / 256 * 256; }

qp_status check_layout(const qp_layout* L) {
  if (L == nullptr) return QP_ERR_INVALID_ARG;
  if (L->n_q_heads <= 0 || L->n_kv_heads <= 0 || L->head_dim <= 0) return QP_ERR_INVALID_ARG;
  if (L->n_q_heads % L->n_kv_heads != 0) return QP_ERR_INVALID_ARG;
  if (L->dtype != QP_F32 && L->dtype != QP_BF16) return QP_ERR_INVALID_ARG;
  if (!(L->softmax_scale >= 0.f) || isinf(L->softmax_scale)) return QP_ERR_INVALID_ARG;
  if (L->head_dim != 64 && L->head_dim != 128) return QP_ERR_UNSUPPORTED;
  if (L->n_q_heads > 65535 || L->n_kv_heads > 65535) return QP_ERR_UNSUPPORTED;
  return QP_OK;
}

qp_status check_group(int32_t n_g) {
  if (n_g <= 0) return QP_ERR_INVALID_ARG;
  if (n_g > QP_MAX_GROUP_TOKENS) return QP_ERR_UNSUPPORTED;
  return QP_OK;
}

qp_status check_cache(const qp_layout* L, const qp_cache* c, bool required) {
  if (c == nullptr) return required ? QP_ERR_INVALID_ARG : QP_OK;
  if (c->capacity < 0 || c->len < 0 || c->len > c->capacity) return QP_ERR_INVALID_ARG;
  if (c->format != QP_CACHE_SAME && c->format != QP_CACHE_FP8_E4M3) return QP_ERR_INVALID_ARG;
  if (c->format == QP_CACHE_FP8_E4M3 && (L->dtype != QP_BF16 || L->head_dim != 128)) return QP_ERR_UNSUPPORTED;
  if (c->len > 0 || required) {
    if (c->k == nullptr || c->v == nullptr || !aligned16(c->k) || !aligned16(c->v)) return QP_ERR_INVALID_ARG;
  }
  if (required && (c->pos == nullptr || (((uintptr_t)c->pos) & 3u))) return QP_ERR_INVALID_ARG;
  return QP_OK;
}

float scale_log2_of(const qp_layout* L) {
  const float scale = L->softmax_scale > 0.f ? L->softmax_scale : 1.0f / sqrtf((float)L->head_dim);
  return scale * 1.4426950408889634f;
}

// Fault injection for the tests of the error paths (qp_debug_fail_after): the n-th status check from now reports a
// launch failure although nothing failed on the GPU. 0 = off.
std::atomic<int> g_fail_countdown{0};

qp_status finish(hipError_t launch_err) {
  hipError_t e = launch_err != hipSuccess ? launch_err : hipGetLastError();
  if (e == hipSuccess && g_fail_countdown.load(std::memory_order_relaxed) > 0 &&
      g_fail_countdown.fetch_sub(1, std::memory_order_relaxed) == 1)
    e = hipErrorLaunchFailure;
  if (e != hipSuccess) {
    g_last_hip_error = (int)e;
    return QP_ERR_HIP;
  }
  return QP_OK;
}

// Scratch of qp_group_attend_noalloc: one array per GPU that the library is loaded on, held until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; the device address it yields (one per
// device) is what launches and copies use.
constexpr size_t kStaticScratchBytes = (size_t)QP_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[qp::QP_MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up once per device), nullptr + status on failure.
qp_status static_scratch(void** out) {
  const int dev = qp::current_device();
  if (dev < 0) return QP_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      g_last_hip_error = (int)(e != hipSuccess ? e : hipErrorInvalidSymbol);
      return QP_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return QP_OK;
}

// Scratch that qp_group_attend's key split may use (partial outputs of the chunks); qp_prefill_video keeps one
// area per attention stream, so that two groups' attention launches in flight never share one.
constexpr size_t kAttendSplitBytes = (size_t)128 << 20;

// Library-owned streams of qp_prefill_video (created once per device, default priority):
//   score   scoring and top-k/compaction of a group depend only on the group's K/V (and the query window),
//           never on its attention, so they run beside the group's attention kernel;
//   attend  the attention of group g+1 depends on the compaction of group g but not on the attention of
//           group g, so consecutive groups' attention kernels alternate between the caller's stream and a
//           second attention stream: launch gaps and the tail of one group's kernel are filled by the next.
// They are forked from the caller's stream at entry and joined back into it before the call returns. The
// streams and their events are shared by all calls on a device, so qp_prefill_video holds g_prefill_mutex while
// it enqueues (it never waits for the GPU inside).
constexpr int MAX_ATT_STREAMS = 2;  // attention streams in rotation, the caller's included (3 measured no better, 4 worse)
struct SideStreams {
  hipStream_t score = nullptr, attend[MAX_ATT_STREAMS] = {};  // attend[0] is unused (the caller's stream)
  hipEvent_t fork = nullptr, compacted[2] = {nullptr, nullptr}, attend_done[MAX_ATT_STREAMS] = {};
  int n_att = MAX_ATT_STREAMS;
  bool tried = false, ok = false;
};
SideStreams g_side_of[qp::QP_MAX_DEVICES];
std::mutex g_prefill_mutex;

// The current device's side streams, created on first use; nullptr if there is no usable device slot or the
// creation failed (the call then runs everything on the caller's stream).
SideStreams* side_streams() {
  const int dev = qp::current_device();
  if (dev < 0) return nullptr;
  SideStreams& g = g_side_of[dev];
  if (!g.tried) {
    g.tried = true;
    g.ok = hipStreamCreateWithFlags(&g.score, hipStreamNonBlocking) == hipSuccess &&
           hipEventCreateWithFlags(&g.fork, hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&g.compacted[0], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&g.compacted[1], hipEventDisableTiming) == hipSuccess;
    for (int i = 1; i < MAX_ATT_STREAMS && g.ok; ++i)
      g.ok = hipStreamCreateWithFlags(&g.attend[i], hipStreamNonBlocking) == hipSuccess &&
             hipEventCreateWithFlags(&g.attend_done[i], hipEventDisableTiming) == hipSuccess;
    if (!g.ok) (void)hipGetLastError();
  }
  return g.ok ? &g : nullptr;
}

// Workspace layout of qp_prefill_video: [scores H_kv*n_g f32][kept indices H_kv*n_g i32][scoring scratch] ... and, at
// the end, one key-split area of kAttendSplitBytes per attention stream.
size_t scores_bytes(const qp_layout* L, int32_t n_g) { return round256((size_t)L->n_kv_heads * n_g * sizeof(float)); }

}  // namespace

namespace qp {

void note_hip_error(int e) { g_last_hip_error = e; }

// Fork/join onto the device's library-owned scoring stream, for callers outside this file that have work which
// may run beside the caller's stream. side_fork orders the side stream after everything enqueued on `main` so far
// and returns it holding the enqueue mutex (the streams and events are shared by all calls on a device); side_join
// makes `main` wait for the side stream and releases the mutex. nullptr: no side stream, nothing is held.
hipStream_t side_fork(hipStream_t main) {
  g_prefill_mutex.lock();
  SideStreams* side = side_streams();
  if (side == nullptr || hipEventRecord(side->fork, main) != hipSuccess ||
      hipStreamWaitEvent(side->score, side->fork, 0) != hipSuccess) {
    (void)hipGetLastError();
    g_prefill_mutex.unlock();
    return nullptr;
  }
  return side->score;
}

void side_join(hipStream_t main) {
  SideStreams* side = side_streams();
  if (side != nullptr) {
    if (hipEventRecord(side->compacted[0], side->score) != hipSuccess ||
        hipStreamWaitEvent(main, side->compacted[0], 0) != hipSuccess)
      (void)hipGetLastError();
  }
  g_prefill_mutex.unlock();
}

int current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return -1;
  }
  return dev >= 0 && dev < QP_MAX_DEVICES ? dev : -1;
}

int device_cu_count() {
  static int cached[QP_MAX_DEVICES] = {};
  const int dev = current_device();
  if (dev < 0) return 256;
  if (cached[dev] == 0) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) {
      (void)hipGetLastError();
      v = 256;
    }
    cached[dev] = v;
  }
  return cached[dev];
}

}  // namespace qp

extern "C" {

int64_t qp_keep_count(int64_t n, double retention) {
  if (!(retention > 0.0) || retention > 1.0) return -1;
  if (n <= 0) return 0;
  int64_t k = (int64_t)ceil(retention * (double)n - 1e-9);
  if (k < 1) k = 1;
  if (k > n) k = n;
  return k;
}

int64_t qp_cache_capacity(int32_t n_frames, int32_t tokens_per_frame, int32_t group_frames, double retention) {
  if (n_frames <= 0 || tokens_per_frame <= 0 || group_frames <= 0) return -1;
  if (!(retention > 0.0) || retention > 1.0) return -1;
  int64_t total = 0;
  for (int64_t f = 0; f < n_frames; f += group_frames) {
    const int64_t g = (n_frames - f) < group_frames ? (n_frames - f) : group_frames;
    total += qp_keep_count(g * tokens_per_frame, retention);
  }
  return total;
}

int32_t qp_group_bounds(int32_t n_frames, int32_t tokens_per_frame, int32_t group_frames, int32_t* first_token,
                        int32_t* n_tokens, int32_t max_groups) {
  if (n_frames <= 0 || tokens_per_frame <= 0 || group_frames <= 0 || max_groups < 0) return -1;
  if ((int64_t)n_frames * tokens_per_frame > INT32_MAX) return -1;
  int32_t gi = 0;
  for (int32_t f = 0; f < n_frames; ++gi) {
    const int32_t g = (n_frames - f) < group_frames ? (n_frames - f) : group_frames;
    if (gi < max_groups) {
      if (first_token != nullptr) first_token[gi] = f * tokens_per_frame;
      if (n_tokens != nullptr) n_tokens[gi] = g * tokens_per_frame;
    }
    f += g;
  }
  return gi;
}

uint8_t qp_e4m3_from_bf16(uint16_t bf16_bits) { return (uint8_t)qp::bf16_to_e4m3(bf16_bits); }

uint16_t qp_bf16_from_e4m3(uint8_t code) { return (uint16_t)qp::e4m3_to_bf16(code); }

size_t qp_workspace_bytes(const qp_layout* L, int32_t max_group_tokens, int32_t n_window) {
  if (check_layout(L) != QP_OK || check_group(max_group_tokens) != QP_OK || n_window < 0) return 0;
  size_t b = scores_bytes(L, max_group_tokens);
  b += qp::topk_workspace_bytes(L->n_kv_heads, max_group_tokens);
  const size_t win = qp::window_workspace_bytes(L->n_q_heads, L->n_kv_heads, max_group_tokens, n_window > 0 ? n_window : 1);
  const size_t logit = qp::window_logit_workspace_bytes(L->n_kv_heads, L->head_dim);
  b += win > logit ? win : logit;
  b += MAX_ATT_STREAMS * kAttendSplitBytes;  // key-split scratch of qp_group_attend, one per attention stream of qp_prefill_video
  return b + 256;
}

qp_status qp_attend_plan(const qp_layout* L, int32_t n_g, int32_t cache_len, size_t workspace_bytes,
                         qp_attend_plan_info* out) {
  qp_status st = check_layout(L);
  if (st != QP_OK) return st;
  if ((st = check_group(n_g)) != QP_OK) return st;
  if (cache_len < 0 || out == nullptr) return QP_ERR_INVALID_ARG;
  qp::AttendArgs a;
  memset(&a, 0, sizeof(a));
  a.n_g = n_g;
  a.h_q = L->n_q_heads;
  a.h_kv = L->n_kv_heads;
  a.d = L->head_dim;
  a.c = a.cap = cache_len;
  const bool mfma_ok = qp::attend_mfma_supported(a, L->dtype);
  const int which = g_attend_kernel.load(std::memory_order_relaxed);
  if (which == QP_ATTEND_MFMA && !mfma_ok) return QP_ERR_UNSUPPORTED;
  memset(out, 0, sizeof(*out));
  if (mfma_ok && which != QP_ATTEND_SCALAR) {
    const bool decode = which == QP_ATTEND_AUTO && qp::attend_decode_applies(a, L->dtype);
    const qp::AttendPlan p = decode ? qp::plan_attend_decode(a, workspace_bytes) : qp::plan_attend_mfma(a, workspace_bytes);
    out->kernel = decode ? QP_ATTEND_MFMA_DECODE : QP_ATTEND_MFMA;
    out->workgroups = p.workgroups;
    out->key_chunks = p.n_split;
    out->tiles_per_chunk = p.split_tiles;
    out->mirrored_rows = p.mirrored;
    out->scratch_bytes = p.scratch_bytes;
    out->split_row_blocks = p.split_rb;
  } else {
    out->kernel = QP_ATTEND_SCALAR;
    out->key_chunks = 1;
  }
  return QP_OK;
}

qp_status qp_select_attend_kernel(int32_t which) {
  if (which != QP_ATTEND_AUTO && which != QP_ATTEND_SCALAR && which != QP_ATTEND_MFMA) return QP_ERR_INVALID_ARG;
  g_attend_kernel.store(which, std::memory_order_relaxed);
  return QP_OK;
}

qp_status qp_group_attend_noalloc(const qp_layout* L, const void* q_g, const void* k_g, const void* v_g, int32_t n_g,
                                  const qp_cache* cache, void* out_g, float* lse, void* hip_stream) {
  qp_status st = check_layout(L);
  if (st != QP_OK) return st;
  if ((st = check_group(n_g)) != QP_OK) return st;
  if ((int64_t)n_g * L->n_q_heads > QP_NOALLOC_MAX_ROWS) return QP_ERR_CAPACITY;
  void* ws = nullptr;
  if ((st = static_scratch(&ws)) != QP_OK) return st;
  return qp_group_attend(L, q_g, k_g, v_g, n_g, cache, out_g, lse, ws, kStaticScratchBytes, hip_stream);
}

qp_status qp_group_attend(const qp_layout* L, const void* q_g, const void* k_g, const void* v_g, int32_t n_g,
                          const qp_cache* cache, void* out_g, float* lse, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  qp_status st = check_layout(L);
  if (st != QP_OK) return st;
  if ((st = check_group(n_g)) != QP_OK) return st;
  if ((st = check_cache(L, cache, false)) != QP_OK) return st;
  if (workspace && (((uintptr_t)workspace) & 255u)) return QP_ERR_INVALID_ARG;
  if (!q_g || !k_g || !v_g || !out_g) return QP_ERR_INVALID_ARG;
  if (!aligned16(q_g) || !aligned16(k_g) || !aligned16(v_g) || !aligned16(out_g)) return QP_ERR_INVALID_ARG;
  if (lse && (((uintptr_t)lse) & 3u)) return QP_ERR_INVALID_ARG;

  qp::AttendArgs a{};
  a.q = q_g;
  a.k = k_g;
  a.v = v_g;
  a.c = cache ? cache->len : 0;
  a.cap = cache ? cache->capacity : 0;
  a.ck = a.c > 0 ? cache->k : nullptr;
  a.cv = a.c > 0 ? cache->v : nullptr;
  a.out = out_g;
  a.lse = lse;
  a.n_g = n_g;
  a.h_q = L->n_q_heads;
  a.h_kv = L->n_kv_heads;
  a.d = L->head_dim;
  a.scale_log2 = scale_log2_of(L);
  a.cache_fp8 = cache != nullptr && cache->format == QP_CACHE_FP8_E4M3 && a.c > 0;

  hipStream_t s = (hipStream_t)hip_stream;
  const bool mfma_ok = qp::attend_mfma_supported(a, L->dtype);
  const int which = g_attend_kernel.load(std::memory_order_relaxed);
  if (which == QP_ATTEND_MFMA && !mfma_ok) return QP_ERR_UNSUPPORTED;
  if (a.cache_fp8 && (!mfma_ok || which == QP_ATTEND_SCALAR)) return QP_ERR_UNSUPPORTED;  // only the MFMA kernel reads it
  const size_t ws_bytes = workspace ? workspace_bytes : 0;
  if (mfma_ok && which == QP_ATTEND_AUTO && qp::attend_decode_applies(a, L->dtype))
    qp::launch_attend_decode(a, workspace, ws_bytes, s);
  else if (mfma_ok && which != QP_ATTEND_SCALAR) qp::launch_attend_mfma(a, workspace, ws_bytes, s);
  else qp::launch_attend_scalar(a, L->dtype, s);
  return finish(hipSuccess);
}

qp_status qp_score_kv(const qp_layout* L, qp_score_rule rule, const void* k_g, const void* v_g, int32_t n_g,
                      const void* q_win, int32_t n_window, float* scores, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  qp_status st = check_layout(L);
  if (st != QP_OK) return st;
  if ((st = check_group(n_g)) != QP_OK) return st;
  if (!scores || (((uintptr_t)scores) & 3u)) return QP_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)hip_stream;
  const bool shared = ((int)rule & QP_SCORE_SHARED_HEADS) != 0;
  const int base_rule = (int)rule & ~QP_SCORE_SHARED_HEADS;
  switch (base_rule) {
    case QP_SCORE_KEY_NORM_SMALL:
      if (!k_g || !aligned16(k_g)) return QP_ERR_INVALID_ARG;
      qp::launch_score_norm(k_g, L->dtype, n_g, L->n_kv_heads, L->head_dim, -1.f, scores, s);
      break;
    case QP_SCORE_VALUE_NORM:
      if (!v_g || !aligned16(v_g)) return QP_ERR_INVALID_ARG;
      qp::launch_score_norm(v_g, L->dtype, n_g, L->n_kv_heads, L->head_dim, +1.f, scores, s);
      break;
    case QP_SCORE_WINDOW_ATTN: {
      if (!k_g || !aligned16(k_g) || !q_win || !aligned16(q_win) || n_window <= 0) return QP_ERR_INVALID_ARG;
      if (n_window > 65535) return QP_ERR_UNSUPPORTED;
      const size_t need = qp::window_workspace_bytes(L->n_q_heads, L->n_kv_heads, n_g, n_window);
      if (!workspace || (((uintptr_t)workspace) & 255u)) return QP_ERR_INVALID_ARG;
      if (workspace_bytes < need) return QP_ERR_CAPACITY;
      qp::WindowArgs w;
      w.k = k_g;
      w.q_win = q_win;
      w.scores = scores;
      w.workspace = workspace;
      w.n_g = n_g;
      w.h_q = L->n_q_heads;
      w.h_kv = L->n_kv_heads;
      w.d = L->head_dim;
      w.w = n_window;
      w.scale_log2 = scale_log2_of(L);
      qp::launch_score_window(w, L->dtype, s);
      break;
    }
    case QP_SCORE_WINDOW_LOGIT: {
      if (!k_g || !aligned16(k_g) || !q_win || !aligned16(q_win) || n_window <= 0) return QP_ERR_INVALID_ARG;
      if (n_window > 65535) return QP_ERR_UNSUPPORTED;
      if (!workspace || (((uintptr_t)workspace) & 255u)) return QP_ERR_INVALID_ARG;
      if (workspace_bytes < qp::window_logit_workspace_bytes(L->n_kv_heads, L->head_dim)) return QP_ERR_CAPACITY;
      qp::WindowArgs w;
      w.k = k_g;
      w.q_win = q_win;
      w.scores = scores;
      w.workspace = workspace;
      w.n_g = n_g;
      w.h_q = L->n_q_heads;
      w.h_kv = L->n_kv_heads;
      w.d = L->head_dim;
      w.w = n_window;
      w.scale_log2 = scale_log2_of(L);
      qp::launch_score_window_logit(w, L->dtype, scale_log2_of(L) * 0.6931471805599453f, s);
      break;
    }
    default:
      return QP_ERR_INVALID_ARG;
  }
  if (shared) qp::launch_share_heads(scores, L->n_kv_heads, n_g, s);
  return finish(hipSuccess);
}

qp_status qp_topk_compact(const qp_layout* L, const float* scores, const void* k_g, const void* v_g, int32_t n_g,
                          int32_t keep, int32_t group_token_base, qp_cache* cache, int32_t* kept_idx, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  qp_status st = check_layout(L);
  if (st != QP_OK) return st;
  if ((st = check_group(n_g)) != QP_OK) return st;
  if ((st = check_cache(L, cache, true)) != QP_OK) return st;
  if (!scores || (((uintptr_t)scores) & 3u) || !k_g || !v_g || !aligned16(k_g) || !aligned16(v_g))
    return QP_ERR_INVALID_ARG;
  if (kept_idx && (((uintptr_t)kept_idx) & 3u)) return QP_ERR_INVALID_ARG;
  if (keep < 1 || keep > n_g || group_token_base < 0) return QP_ERR_INVALID_ARG;
  if ((int64_t)cache->len + keep > cache->capacity) return QP_ERR_CAPACITY;
  (void)workspace;  // selection and copy are one launch: the kept indices never leave the kernel unless asked for
  (void)workspace_bytes;

  qp::TopkArgs a;
  a.scores = scores;
  a.k = k_g;
  a.v = v_g;
  a.ck = cache->k;
  a.cv = cache->v;
  a.pos = cache->pos;
  a.n_g = n_g;
  a.h_kv = L->n_kv_heads;
  a.d = L->head_dim;
  a.keep = keep;
  a.base = group_token_base;
  a.cap = cache->capacity;
  a.len = cache->len;
  a.cache_fp8 = cache->format == QP_CACHE_FP8_E4M3;
  st = finish(qp::launch_topk_compact(a, L->dtype, kept_idx, (hipStream_t)hip_stream));
  if (st == QP_OK) cache->len += keep;
  return st;
}

qp_status qp_prefill_video(const qp_layout* L, int32_t n_frames, int32_t tokens_per_frame, int32_t group_frames,
                           double retention, qp_score_rule rule, const void* q, const void* k, const void* v,
                           const void* q_win, int32_t n_window, qp_cache* cache, void* out, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  qp_status st = check_layout(L);
  if (st != QP_OK) return st;
  if (n_frames <= 0 || tokens_per_frame <= 0 || group_frames <= 0) return QP_ERR_INVALID_ARG;
  if (!(retention > 0.0) || retention > 1.0) return QP_ERR_INVALID_ARG;
  const int base_rule = (int)rule & ~QP_SCORE_SHARED_HEADS;
  const bool window_rule = base_rule == QP_SCORE_WINDOW_ATTN || base_rule == QP_SCORE_WINDOW_LOGIT;
  if (base_rule != QP_SCORE_KEY_NORM_SMALL && base_rule != QP_SCORE_VALUE_NORM && !window_rule) return QP_ERR_INVALID_ARG;
  const int64_t n_total = (int64_t)n_frames * tokens_per_frame;
  if (n_total > INT32_MAX) return QP_ERR_UNSUPPORTED;
  const int64_t max_group = (int64_t)(group_frames < n_frames ? group_frames : n_frames) * tokens_per_frame;
  if (max_group > QP_MAX_GROUP_TOKENS) return QP_ERR_UNSUPPORTED;
  if ((st = check_cache(L, cache, true)) != QP_OK) return st;
  if (!q || !k || !v || !out || !aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
    return QP_ERR_INVALID_ARG;
  if (window_rule && (!q_win || !aligned16(q_win) || n_window <= 0)) return QP_ERR_INVALID_ARG;
  if (window_rule && n_window > 65535) return QP_ERR_UNSUPPORTED;
  if (!workspace || (((uintptr_t)workspace) & 255u)) return QP_ERR_INVALID_ARG;
  if (workspace_bytes < qp_workspace_bytes(L, (int32_t)max_group, window_rule ? n_window : 0))
    return QP_ERR_CAPACITY;
  if ((int64_t)cache->len + qp_cache_capacity(n_frames, tokens_per_frame, group_frames, retention) > cache->capacity)
    return QP_ERR_CAPACITY;
  if (g_attend_kernel.load(std::memory_order_relaxed) == QP_ATTEND_MFMA) {
    qp::AttendArgs probe;
    memset(&probe, 0, sizeof(probe));
    probe.h_q = L->n_q_heads;
    probe.h_kv = L->n_kv_heads;
    probe.d = L->head_dim;
    probe.n_g = (int)max_group;
    if (!qp::attend_mfma_supported(probe, L->dtype)) return QP_ERR_UNSUPPORTED;
  }

  const size_t esz = L->dtype == QP_F32 ? 4 : 2;
  const size_t q_tok = (size_t)L->n_q_heads * L->head_dim * esz;
  const size_t kv_tok = (size_t)L->n_kv_heads * L->head_dim * esz;
  float* scores = (float*)workspace;
  const size_t sb = scores_bytes(L, (int32_t)max_group);
  const size_t kb = qp::topk_workspace_bytes(L->n_kv_heads, (int32_t)max_group);
  void* ws2 = (char*)workspace + sb + kb;  // window scratch, then the two key-split areas of the attention streams
  const size_t ws2_bytes = workspace_bytes - sb - kb - MAX_ATT_STREAMS * kAttendSplitBytes;
  char* split_ws = (char*)workspace + (workspace_bytes - MAX_ATT_STREAMS * kAttendSplitBytes) / 256 * 256;

  hipStream_t main_stream = (hipStream_t)hip_stream;
  std::lock_guard<std::mutex> lock(g_prefill_mutex);
  SideStreams* side = side_streams();
  const bool overlap = side != nullptr;
  SideStreams none;
  SideStreams& g_side = overlap ? *side : none;
  void* score_stream = overlap ? (void*)g_side.score : hip_stream;
  // Groups whose attention launch already is several rounds of workgroups gain nothing from a second attention
  // stream (their launches are balanced by the planner, and two of them in flight share the L2s): measured 0.2-1 %
  // faster on one stream from two rounds up, 5 % slower below one round.
  const long group_rows = (long)(group_frames < n_frames ? group_frames : n_frames) * tokens_per_frame * (L->n_q_heads / L->n_kv_heads);
  const long group_wgs = (group_rows + 255) / 256 * L->n_kv_heads;
  const int n_att = !overlap ? 1 : (group_wgs >= 2L * qp::device_cu_count() ? 1 : g_side.n_att);
  // A failed stream call or launch stops the loop (nothing further is enqueued) but never skips the join below.
  const int32_t len_at_entry = cache->len;
#define QP_HIP_OK(call_) \
  if (st == QP_OK && (call_) != hipSuccess) st = finish(hipGetLastError())
  if (overlap) {
    QP_HIP_OK(hipEventRecord(g_side.fork, main_stream));
    QP_HIP_OK(hipStreamWaitEvent(g_side.score, g_side.fork, 0));
    for (int i = 1; i < n_att; ++i) QP_HIP_OK(hipStreamWaitEvent(g_side.attend[i], g_side.fork, 0));
  }
  int gi = 0;
  for (int32_t f = 0; f < n_frames && st == QP_OK; f += group_frames, ++gi) {
    const int32_t g = (n_frames - f) < group_frames ? (n_frames - f) : group_frames;
    const int32_t base = f * tokens_per_frame, n_g = g * tokens_per_frame;
    const char* qg = (const char*)q + (size_t)base * q_tok;
    const char* kg = (const char*)k + (size_t)base * kv_tok;
    const char* vg = (const char*)v + (size_t)base * kv_tok;
    char* og = (char*)out + (size_t)base * q_tok;
    // 1. attend to the pruned cache so far (complete once the previous group's compaction is) + the group itself
    const int ai = gi % n_att;
    hipStream_t att_stream = ai ? g_side.attend[ai] : main_stream;
    if (overlap && gi > 0) QP_HIP_OK(hipStreamWaitEvent(att_stream, g_side.compacted[(gi - 1) & 1], 0));
    if (st != QP_OK) break;
    st = qp_group_attend(L, qg, kg, vg, n_g, cache, og, nullptr, split_ws + ai * kAttendSplitBytes, kAttendSplitBytes,
                         (void*)att_stream);
    if (st != QP_OK) break;
    // 2. score the group's new KV entries; 3. TopK + compaction into the cache (cache->len advances on the host).
    //    The appended rows [len, len+k) are disjoint from the rows [0, len) any attention kernel in flight reads.
    const int32_t keep = (int32_t)qp_keep_count(n_g, retention);
    if (keep < n_g) {  // at retention 1 every token survives whatever its score
      st = qp_score_kv(L, rule, kg, vg, n_g, q_win, n_window, scores, ws2, ws2_bytes, score_stream);
      if (st != QP_OK) break;
    }
    st = qp_topk_compact(L, scores, kg, vg, n_g, keep, base, cache, nullptr, ws2, ws2_bytes, score_stream);
    if (st != QP_OK) break;
    if (overlap) QP_HIP_OK(hipEventRecord(g_side.compacted[gi & 1], g_side.score));
  }
#undef QP_HIP_OK
  // Join, on success and on failure alike: everything enqueued on the library's streams is ordered before whatever
  // the caller enqueues next on hip_stream. A join call that fails is reported unless an earlier error already is.
  if (overlap) {
    hipError_t je = hipEventRecord(g_side.compacted[0], g_side.score);
    if (je == hipSuccess) je = hipStreamWaitEvent(main_stream, g_side.compacted[0], 0);
    for (int i = 1; i < n_att; ++i) {
      hipError_t e = hipEventRecord(g_side.attend_done[i], g_side.attend[i]);
      if (e == hipSuccess) e = hipStreamWaitEvent(main_stream, g_side.attend_done[i], 0);
      if (je == hipSuccess) je = e;
    }
    if (je != hipSuccess) {
      const qp_status js = finish(je);
      if (st == QP_OK) st = js;
    }
  }
  // After a failure the groups already enqueued still run, but the cache is handed back at its length at entry:
  // rows beyond it are scratch.
  if (st != QP_OK) cache->len = len_at_entry;
  return st;
}

qp_status qp_debug_fail_after(int32_t n_checks) {
  if (n_checks < 0) return QP_ERR_INVALID_ARG;
  g_fail_countdown.store(n_checks, std::memory_order_relaxed);
  return QP_OK;
}

const char* qp_status_string(qp_status s) {
  switch ((int)s) {  // callers across the C ABI may pass any int
    case QP_OK: return "ok";
    case QP_ERR_INVALID_ARG: return "invalid argument";
    case QP_ERR_UNSUPPORTED: return "unsupported dtype, head_dim or size";
    case QP_ERR_CAPACITY: return "cache capacity or workspace too small";
    case QP_ERR_HIP: return "HIP launch failed";
    case QP_FEED_END: return "feed closed and drained";
    case QP_FEED_TIMEOUT: return "nothing published within the time-out";
  }
  return "unknown status";
}

int qp_last_hip_error(void) { return g_last_hip_error; }

const char* qp_version(void) { return "quickprefill-gfx950 0.1"; }

}  // extern "C"
