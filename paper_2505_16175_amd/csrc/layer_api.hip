// C-ABI entry points of the decoder layer around the path (qp_layer.h): validation, workspace carving, launches.
// Host code only.
#include <math.h>

#include "qp_internal.h"
#include "qp_layer.h"

namespace {

inline bool aligned16(const void* p) { return p != nullptr && (((uintptr_t)p) & 15u) == 0; }
inline size_t round256(size_t x) { return (x + 255) / 256 * 256; }

qp_status finish(hipError_t launch_err) {
  hipError_t e = launch_err != hipSuccess ? launch_err : hipGetLastError();
  if (e != hipSuccess) {
    qp::note_hip_error((int)e);
    return QP_ERR_HIP;
  }
  return QP_OK;
}

qp_status check_layer(const qp_layout* L, const qp_layer_shape* S) {
  if (L == nullptr || S == nullptr) return QP_ERR_INVALID_ARG;
  if (L->n_q_heads <= 0 || L->n_kv_heads <= 0 || L->n_q_heads % L->n_kv_heads != 0) return QP_ERR_INVALID_ARG;
  if (S->d_model <= 0 || S->d_ff <= 0 || !(S->rms_eps >= 0.f) || !(S->rope_theta > 0.f)) return QP_ERR_INVALID_ARG;
  for (int a = 0; a < 3; ++a)
    if (S->mrope_section[a] < 0) return QP_ERR_INVALID_ARG;
  if (L->dtype != QP_BF16 || L->head_dim != 128) return QP_ERR_UNSUPPORTED;
  if (S->mrope_section[0] + S->mrope_section[1] + S->mrope_section[2] != 64) return QP_ERR_INVALID_ARG;
  if (S->d_model % 64 != 0 || S->d_ff % 128 != 0 || (L->n_q_heads + 2 * L->n_kv_heads) % 2 != 0) return QP_ERR_UNSUPPORTED;
  return QP_OK;
}

// Workspace of qp_layer_group, in order: h | q | k | v | attn | x1 | act | cos_sin | scores | projection split
// scratch | path workspace
// Room for the partial sums of a split contraction (launches of few tokens; see gemm_plan_split)
constexpr size_t kGemmSplitBytes = (size_t)32 << 20;

struct Carve {
  size_t h, q, k, v, attn, x1, act, cs, scores, gemm, path, total;
};
Carve carve(const qp_layout* L, const qp_layer_shape* S, int32_t n_g, int32_t n_window) {
  Carve c{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += round256(bytes);
    return at;
  };
  c.h = take((size_t)n_g * S->d_model * 2);
  c.q = take((size_t)n_g * L->n_q_heads * 128 * 2);
  c.k = take((size_t)n_g * L->n_kv_heads * 128 * 2);
  c.v = take((size_t)n_g * L->n_kv_heads * 128 * 2);
  c.attn = take((size_t)n_g * L->n_q_heads * 128 * 2);
  c.x1 = take((size_t)n_g * S->d_model * 2);
  c.act = take((size_t)n_g * S->d_ff * 2);
  c.cs = take((size_t)n_g * 64 * 2 * sizeof(float));
  c.scores = take((size_t)L->n_kv_heads * n_g * sizeof(float));
  c.gemm = take(kGemmSplitBytes);
  c.path = off;
  c.total = off + qp_workspace_bytes(L, n_g, n_window);
  return c;
}

}  // namespace

extern "C" {

qp_status qp_rms_norm(const void* x, const void* w, void* out, int32_t n_tokens, int32_t d_model, float eps,
                      void* hip_stream) {
  if (!aligned16(x) || !aligned16(w) || !aligned16(out) || n_tokens <= 0 || d_model <= 0 || !(eps >= 0.f))
    return QP_ERR_INVALID_ARG;
  if (d_model % 8 != 0) return QP_ERR_UNSUPPORTED;
  qp::launch_rms_norm(x, w, out, n_tokens, d_model, eps, (hipStream_t)hip_stream);
  return finish(hipSuccess);
}

qp_status qp_linear(const void* x, const void* w, const void* bias_or_null, const void* residual_or_null, void* out,
                    int32_t m, int32_t n, int32_t k, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!aligned16(x) || !aligned16(w) || !aligned16(out) || m <= 0 || n <= 0 || k <= 0) return QP_ERR_INVALID_ARG;
  if (workspace != nullptr && (((uintptr_t)workspace) & 255u)) return QP_ERR_INVALID_ARG;
  if ((bias_or_null != nullptr && !aligned16(bias_or_null)) || (residual_or_null != nullptr && !aligned16(residual_or_null)))
    return QP_ERR_INVALID_ARG;
  qp::GemmArgs a{};
  a.x = x, a.w = w, a.bias = bias_or_null, a.residual = residual_or_null, a.out = out;
  a.m = m, a.n = n, a.k = k;
  if (!qp::gemm_supported(a, qp::GEMM_PLAIN)) return QP_ERR_UNSUPPORTED;
  return finish(qp::launch_gemm_bf16(a, qp::GEMM_PLAIN, workspace, workspace_bytes, (hipStream_t)hip_stream));
}

qp_status qp_rope_table(const int32_t* pos, int64_t axis_stride, int32_t n_tokens, float theta,
                        const int32_t mrope_section[3], float* cos_sin, void* hip_stream) {
  if (pos == nullptr || (((uintptr_t)pos) & 3u) || !aligned16(cos_sin) || n_tokens <= 0 || axis_stride < 0 ||
      !(theta > 0.f) || mrope_section == nullptr)
    return QP_ERR_INVALID_ARG;
  if (mrope_section[0] < 0 || mrope_section[1] < 0 || mrope_section[2] < 0 ||
      mrope_section[0] + mrope_section[1] + mrope_section[2] != 64)
    return QP_ERR_INVALID_ARG;
  if (n_tokens > QP_MAX_GROUP_TOKENS) return QP_ERR_UNSUPPORTED;
  qp::launch_rope_table(pos, (long)axis_stride, n_tokens, theta, mrope_section[0], mrope_section[1], cos_sin,
                        (hipStream_t)hip_stream);
  return finish(hipSuccess);
}

qp_status qp_qkv_rope(const qp_layout* layout, const void* h, const void* w_qkv, const void* b_qkv,
                      const float* cos_sin, int32_t n_tokens, int32_t d_model, void* q, void* k, void* v,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (layout == nullptr || layout->n_q_heads <= 0 || layout->n_kv_heads <= 0) return QP_ERR_INVALID_ARG;
  if (workspace != nullptr && (((uintptr_t)workspace) & 255u)) return QP_ERR_INVALID_ARG;
  if (!aligned16(h) || !aligned16(w_qkv) || !aligned16(b_qkv) || !aligned16(cos_sin) || !aligned16(q) ||
      !aligned16(k) || !aligned16(v) || n_tokens <= 0 || d_model <= 0)
    return QP_ERR_INVALID_ARG;
  if (layout->dtype != QP_BF16 || layout->head_dim != 128) return QP_ERR_UNSUPPORTED;
  qp::GemmArgs a{};
  a.x = h, a.w = w_qkv, a.bias = b_qkv, a.q = q, a.k_out = k, a.v_out = v, a.cos_sin = cos_sin;
  a.m = n_tokens, a.n = (layout->n_q_heads + 2 * layout->n_kv_heads) * 128, a.k = d_model;
  a.h_q = layout->n_q_heads, a.h_kv = layout->n_kv_heads;
  if (!qp::gemm_supported(a, qp::GEMM_QKV_ROPE)) return QP_ERR_UNSUPPORTED;
  return finish(qp::launch_gemm_bf16(a, qp::GEMM_QKV_ROPE, workspace, workspace_bytes, (hipStream_t)hip_stream));
}

qp_status qp_swiglu_gate_up(const void* h, const void* w_gate_up, void* act, int32_t n_tokens, int32_t d_model,
                            int32_t d_ff, void* hip_stream) {
  if (!aligned16(h) || !aligned16(w_gate_up) || !aligned16(act) || n_tokens <= 0 || d_model <= 0 || d_ff <= 0)
    return QP_ERR_INVALID_ARG;
  if (d_ff > (1 << 29)) return QP_ERR_UNSUPPORTED;
  qp::GemmArgs a{};
  a.x = h, a.w = w_gate_up, a.out = act;
  a.m = n_tokens, a.n = 2 * d_ff, a.k = d_model;
  if (!qp::gemm_supported(a, qp::GEMM_SWIGLU)) return QP_ERR_UNSUPPORTED;
  return finish(qp::launch_gemm_bf16(a, qp::GEMM_SWIGLU, nullptr, 0, (hipStream_t)hip_stream));
}

qp_status qp_linear_plan(int32_t m, int32_t n, int32_t k, size_t workspace_bytes, qp_linear_plan_info* out) {
  if (out == nullptr || m <= 0 || n <= 0 || k <= 0) return QP_ERR_INVALID_ARG;
  qp::GemmArgs a{};
  a.m = m, a.n = n, a.k = k;
  if (!qp::gemm_supported(a, qp::GEMM_PLAIN)) return QP_ERR_UNSUPPORTED;
  const qp::GemmSplit sp = qp::gemm_plan_split(a, qp::GEMM_PLAIN, workspace_bytes);
  if (qp::gemm_uses_gemv(a)) {  // the weight-streaming kernel: 4 weight rows per workgroup, never split
    out->token_rows_per_tile = m;
    out->workgroups = n / 4;
    out->k_chunks = 1;
    out->k_steps_per_chunk = sp.steps_per_split;
    out->scratch_bytes = 0;
    return QP_OK;
  }
  const int rows = qp::gemm_tile_rows(a);
  const int tiles_m = (m + rows - 1) / rows, tiles_n = (n + 255) / 256;
  const int m_block = tiles_m < 8 ? tiles_m : 8;
  out->token_rows_per_tile = rows;
  out->workgroups = 8 * ((tiles_m + m_block - 1) / m_block) * m_block * (((tiles_n + 7) / 8 + 3) / 4) * 4;
  out->k_chunks = sp.split_k;
  out->k_steps_per_chunk = sp.steps_per_split;
  out->scratch_bytes = sp.scratch_bytes;
  return QP_OK;
}

qp_status qp_select_linear_tile(int32_t token_rows) {
  if (token_rows != 0 && token_rows != 128 && token_rows != 256) return QP_ERR_INVALID_ARG;
  qp::gemm_force_tile_rows(token_rows);
  return QP_OK;
}

size_t qp_layer_workspace_bytes(const qp_layout* layout, const qp_layer_shape* shape, int32_t max_group_tokens,
                                int32_t n_window) {
  if (check_layer(layout, shape) != QP_OK || max_group_tokens <= 0 || max_group_tokens > QP_MAX_GROUP_TOKENS ||
      n_window < 0)
    return 0;
  const int32_t n = max_group_tokens > n_window ? max_group_tokens : n_window;
  if (qp_workspace_bytes(layout, n, n_window) == 0) return 0;
  return carve(layout, shape, n, n_window).total;
}

qp_status qp_layer_group(const qp_layout* layout, const qp_layer_shape* shape, const qp_layer_weights* weights,
                         const void* x_g, const int32_t* pos, int64_t axis_stride, int32_t n_group_tokens,
                         int32_t group_token_base, const void* q_win, int32_t n_window, qp_score_rule rule,
                         int32_t keep, qp_cache* cache, void* x_out, int32_t* kept_idx_or_null, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  qp_status st = check_layer(layout, shape);
  if (st != QP_OK) return st;
  if (weights == nullptr || !aligned16(weights->ln1_w) || !aligned16(weights->w_qkv) || !aligned16(weights->b_qkv) ||
      !aligned16(weights->w_o) || !aligned16(weights->ln2_w) || !aligned16(weights->w_gate_up) ||
      !aligned16(weights->w_down))
    return QP_ERR_INVALID_ARG;
  if (!aligned16(x_g) || !aligned16(x_out) || pos == nullptr || (((uintptr_t)pos) & 3u) || axis_stride < 0 ||
      cache == nullptr || workspace == nullptr || (((uintptr_t)workspace) & 255u))
    return QP_ERR_INVALID_ARG;
  if (n_group_tokens <= 0 || group_token_base < 0 || n_window < 0) return QP_ERR_INVALID_ARG;
  if (n_group_tokens > QP_MAX_GROUP_TOKENS) return QP_ERR_UNSUPPORTED;
  if (keep < 1 || keep > n_group_tokens) return QP_ERR_INVALID_ARG;
  const int base_rule = (int)rule & 0xff;
  const bool windowed = base_rule == QP_SCORE_WINDOW_ATTN || base_rule == QP_SCORE_WINDOW_LOGIT;
  if (base_rule > QP_SCORE_WINDOW_LOGIT || ((int)rule & ~(0xff | QP_SCORE_SHARED_HEADS))) return QP_ERR_INVALID_ARG;
  if (windowed && (!aligned16(q_win) || n_window <= 0)) return QP_ERR_INVALID_ARG;
  if (cache->capacity < 0 || cache->len < 0 || cache->len > cache->capacity || !aligned16(cache->k) ||
      !aligned16(cache->v) || cache->pos == nullptr)
    return QP_ERR_INVALID_ARG;
  if ((int64_t)cache->len + keep > cache->capacity) return QP_ERR_CAPACITY;
  const int32_t nw = windowed ? n_window : 0;
  const Carve c = carve(layout, shape, n_group_tokens, nw);
  if (workspace_bytes < c.total) return QP_ERR_CAPACITY;

  // every projection's shape is checked before the first launch
  const int n_g = n_group_tokens, dm = shape->d_model, hq = layout->n_q_heads, hkv = layout->n_kv_heads;
  unsigned char* ws = (unsigned char*)workspace;
  qp::GemmArgs qkv{}, oproj{}, gate_up{}, down{};
  qkv.x = ws + c.h, qkv.w = weights->w_qkv, qkv.bias = weights->b_qkv, qkv.q = ws + c.q, qkv.k_out = ws + c.k,
  qkv.v_out = ws + c.v, qkv.cos_sin = (const float*)(ws + c.cs);
  qkv.m = n_g, qkv.n = (hq + 2 * hkv) * 128, qkv.k = dm, qkv.h_q = hq, qkv.h_kv = hkv;
  oproj.x = ws + c.attn, oproj.w = weights->w_o, oproj.residual = x_g, oproj.out = ws + c.x1;
  oproj.m = n_g, oproj.n = dm, oproj.k = hq * 128;
  gate_up.x = ws + c.h, gate_up.w = weights->w_gate_up, gate_up.out = ws + c.act;
  gate_up.m = n_g, gate_up.n = 2 * shape->d_ff, gate_up.k = dm;
  down.x = ws + c.act, down.w = weights->w_down, down.residual = ws + c.x1, down.out = x_out;
  down.m = n_g, down.n = dm, down.k = shape->d_ff;
  if (!qp::gemm_supported(qkv, qp::GEMM_QKV_ROPE) || !qp::gemm_supported(oproj, qp::GEMM_PLAIN) ||
      !qp::gemm_supported(gate_up, qp::GEMM_SWIGLU) || !qp::gemm_supported(down, qp::GEMM_PLAIN))
    return QP_ERR_UNSUPPORTED;

  hipStream_t s = (hipStream_t)hip_stream;
  // path workspace: the key-split scratch of the attention at its end, scoring / top-k scratch at its start
  constexpr size_t kSplit = (size_t)32 << 20;
  const size_t path_bytes = workspace_bytes - c.path;
  void* score_ws = ws + c.path;
  const size_t score_bytes = path_bytes - kSplit;
  void* split_ws = ws + c.path + (path_bytes - kSplit) / 256 * 256;
  qp::launch_rms_norm(x_g, weights->ln1_w, ws + c.h, n_g, dm, shape->rms_eps, s);
  qp::launch_rope_table(pos, (long)axis_stride, n_g, shape->rope_theta, shape->mrope_section[0], shape->mrope_section[1],
                        (float*)(ws + c.cs), s);
  st = finish(qp::launch_gemm_bf16(qkv, qp::GEMM_QKV_ROPE, ws + c.gemm, kGemmSplitBytes, s));
  if (st != QP_OK) return st;
  // Scoring, top-k and compaction need the group's K and V only, not its attention: they run on the library's side
  // stream beside the attention and the projections that follow, and are joined back before the call returns.
  // The attention reads cache entries [0, len), the compaction writes [len, len + keep).
  struct Side {
    hipStream_t main, side;
    explicit Side(hipStream_t m) : main(m), side(qp::side_fork(m)) {}
    ~Side() {
      if (side != nullptr) qp::side_join(main);
    }
    hipStream_t stream() const { return side != nullptr ? side : main; }
  } fork(s);
  st = qp_group_attend(layout, ws + c.q, ws + c.k, ws + c.v, n_g, cache, ws + c.attn, nullptr, split_ws, kSplit, s);
  if (st != QP_OK) return st;
  if (keep < n_g) {  // with every token kept (the stages after the video) the scores decide nothing
    st = qp_score_kv(layout, rule, ws + c.k, ws + c.v, n_g, q_win, nw, (float*)(ws + c.scores), score_ws, score_bytes,
                     fork.stream());
    if (st != QP_OK) return st;
  }
  st = qp_topk_compact(layout, (const float*)(ws + c.scores), ws + c.k, ws + c.v, n_g, keep, group_token_base, cache,
                       kept_idx_or_null, score_ws, score_bytes, fork.stream());
  if (st != QP_OK) return st;
  st = finish(qp::launch_gemm_bf16(oproj, qp::GEMM_PLAIN, ws + c.gemm, kGemmSplitBytes, s));
  if (st != QP_OK) return st;
  qp::launch_rms_norm(ws + c.x1, weights->ln2_w, ws + c.h, n_g, dm, shape->rms_eps, s);
  st = finish(qp::launch_gemm_bf16(gate_up, qp::GEMM_SWIGLU, nullptr, 0, s));
  if (st != QP_OK) return st;
  return finish(qp::launch_gemm_bf16(down, qp::GEMM_PLAIN, ws + c.gemm, kGemmSplitBytes, s));
}

qp_status qp_layer_window_queries(const qp_layout* layout, const qp_layer_shape* shape,
                                  const qp_layer_weights* weights, const void* x_win, const int32_t* pos,
                                  int64_t axis_stride, int32_t n_window, void* q_win_out, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  qp_status st = check_layer(layout, shape);
  if (st != QP_OK) return st;
  if (weights == nullptr || !aligned16(weights->ln1_w) || !aligned16(weights->w_qkv) || !aligned16(weights->b_qkv))
    return QP_ERR_INVALID_ARG;
  if (!aligned16(x_win) || !aligned16(q_win_out) || pos == nullptr || (((uintptr_t)pos) & 3u) || axis_stride < 0 ||
      workspace == nullptr || (((uintptr_t)workspace) & 255u) || n_window <= 0)
    return QP_ERR_INVALID_ARG;
  if (n_window > QP_MAX_GROUP_TOKENS) return QP_ERR_UNSUPPORTED;
  const Carve c = carve(layout, shape, n_window, n_window);
  if (workspace_bytes < c.total) return QP_ERR_CAPACITY;
  unsigned char* ws = (unsigned char*)workspace;
  // the window's keys and values are by-products of the fused projection; they land in the k / v areas, unused
  qp::GemmArgs qkv{};
  qkv.x = ws + c.h, qkv.w = weights->w_qkv, qkv.bias = weights->b_qkv, qkv.q = q_win_out, qkv.k_out = ws + c.k,
  qkv.v_out = ws + c.v, qkv.cos_sin = (const float*)(ws + c.cs);
  qkv.m = n_window, qkv.n = (layout->n_q_heads + 2 * layout->n_kv_heads) * 128, qkv.k = shape->d_model;
  qkv.h_q = layout->n_q_heads, qkv.h_kv = layout->n_kv_heads;
  if (!qp::gemm_supported(qkv, qp::GEMM_QKV_ROPE)) return QP_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)hip_stream;
  qp::launch_rms_norm(x_win, weights->ln1_w, ws + c.h, n_window, shape->d_model, shape->rms_eps, s);
  qp::launch_rope_table(pos, (long)axis_stride, n_window, shape->rope_theta, shape->mrope_section[0],
                        shape->mrope_section[1], (float*)(ws + c.cs), s);
  return finish(qp::launch_gemm_bf16(qkv, qp::GEMM_QKV_ROPE, ws + c.gemm, kGemmSplitBytes, s));
}

}  // extern "C"
