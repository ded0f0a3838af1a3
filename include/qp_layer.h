/*
 * qp_layer.h -- C ABI of one decoder layer around the QuickPrefill path, one group at a time (gfx950).
 *
 * Sec. 3.2 of the QuickVideo paper prefills a video group by group so that a transformer block's activations
 * exist for one group only (Appendix D.1 prices the attention block and the SwiGLU MLP block,
 * SwiGLU(x) = W_down(SiLU(W_gate x) * W_up x)). These entry points run the pre-norm decoder layer of the Qwen2.5
 * family the paper evaluates on one group of tokens, with the group attention, scoring, TopK and compaction of
 * qp.h in the middle:
 *     h = RMSNorm(x) ; q,k,v = h W_qkv^T + b_qkv ; rotary embedding on q,k
 *     a = qp_group_attend(q,k,v, this layer's pruned cache) ; qp_score_kv ; qp_topk_compact
 *     x1 = x + a W_o^T ; x_out = x1 + W_down(SiLU(W_gate h2) * W_up h2), h2 = RMSNorm(x1)
 * Keys are rotated before they are cached, so cached keys carry their own positions.
 *
 * Conventions as in qp.h: every data pointer is a DEVICE pointer unless it says host, tensors are dense, row-major
 * and 16-byte aligned, the library allocates nothing, all work is enqueued on `hip_stream`, errors come back as
 * qp_status and are detected on the host before anything is launched.
 * Supported: bf16 activations and weights (f32 accumulation, one rounding to bf16 where a tensor is stored),
 * head_dim 128, d_model and d_ff multiples of 64, d_ff a multiple of 128, (H_q + 2 H_kv) even.
 */
#ifndef QP_LAYER_H_
#define QP_LAYER_H_

#include "qp.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t d_model;          /* hidden size                                                              */
  int32_t d_ff;             /* MLP intermediate size                                                    */
  float rms_eps;            /* RMSNorm: y = x / sqrt(mean(x^2) + eps) * w                               */
  float rope_theta;         /* rotary base: frequency i of head_dim/2 is theta^(-2i/head_dim)           */
  int32_t mrope_section[3]; /* frequencies [0,s0) rotate by the temporal position index, [s0,s0+s1) by the
                               height index, the rest by the width index; s0+s1+s2 = head_dim/2        */
} qp_layer_shape;

/* Weights of one layer, bf16, row-major [out][in] (host struct of device pointers; read only). */
typedef struct {
  const void* ln1_w;     /* [d_model]                                                                    */
  const void* w_qkv;     /* [(H_q + 2 H_kv) * 128][d_model]: query heads, then key heads, then value heads */
  const void* b_qkv;     /* [(H_q + 2 H_kv) * 128]                                                       */
  const void* w_o;       /* [d_model][H_q * 128]                                                         */
  const void* ln2_w;     /* [d_model]                                                                    */
  const void* w_gate_up; /* [2 * d_ff][d_model]: the d_ff gate rows, then the d_ff up rows               */
  const void* w_down;    /* [d_model][d_ff]                                                              */
} qp_layer_weights;

/* ---- the parts (each is one launch) ------------------------------------------------------------------- */

/* out[t][:] = x[t][:] / sqrt(mean(x[t][:]^2) + eps) * w, bf16 [n_tokens][d_model]; d_model a multiple of 8. */
qp_status qp_rms_norm(const void* x, const void* w, void* out, int32_t n_tokens, int32_t d_model, float eps,
                      void* hip_stream);

/* out[m][n] = sum_k x[m][k] w[n][k] (+ bias[n]) (+ residual[m][n]), all bf16, f32 accumulation, one rounding.
 * x [m][k], w [n][k], bias [n] or NULL, residual [m][n] or NULL (may alias out), out [m][n].
 *   workspace: optional device scratch (256-byte aligned), may be NULL. A call whose output tiles would occupy at
 *     most a quarter of the compute units (few tokens against long rows: text chunks, decode steps, where streaming
 *     the weights once is the bound) deals the contraction to k chunks, about one workgroup per compute unit in
 *     all; their f32 partial sums ([chunks][m][n], as many chunks as fit) live in this scratch and a second launch
 *     adds them in chunk order and applies bias / residual. Without scratch nothing is split. Same inputs, same
 *     scratch size: bit-identical results.
 * UNSUPPORTED unless k is a multiple of 64 and n a multiple of 8. */
qp_status qp_linear(const void* x, const void* w, const void* bias_or_null, const void* residual_or_null, void* out,
                    int32_t m, int32_t n, int32_t k, void* workspace, size_t workspace_bytes, void* hip_stream);

/* cos_sin[t][i] = (cos, sin)(pos[axis(i)][t] * theta^(-i/64)), f32 [n_tokens][64][2], for head_dim 128.
 * pos: int32, position index of token t on axis a at pos[a * axis_stride + t] (a = 0 temporal, 1 height, 2 width),
 * so a group is a pointer into a [3][N] array with axis_stride = N. */
qp_status qp_rope_table(const int32_t* pos, int64_t axis_stride, int32_t n_tokens, float theta,
                        const int32_t mrope_section[3], float* cos_sin, void* hip_stream);

/* q, k, v = h w_qkv^T + b_qkv split into heads, rotary embedding applied to q and k (pairs (i, i+64) of a head),
 * written token-major: q [n_tokens][H_q][128], k, v [n_tokens][H_kv][128]. h [n_tokens][d_model].
 * workspace: as in qp_linear (the rotary embedding then runs in the second launch). */
qp_status qp_qkv_rope(const qp_layout* layout, const void* h, const void* w_qkv, const void* b_qkv,
                      const float* cos_sin, int32_t n_tokens, int32_t d_model, void* q, void* k, void* v,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* act = SiLU(h w_gate^T) * (h w_up^T), bf16 [n_tokens][d_ff] (Appendix D.1); gate and up never reach memory. */
qp_status qp_swiglu_gate_up(const void* h, const void* w_gate_up, void* act, int32_t n_tokens, int32_t d_model,
                            int32_t d_ff, void* hip_stream);

/* The projections run 256 x 256 output tiles per workgroup, or 128 (tokens) x 256 when the larger tile would leave
 * compute units idle; the launcher chooses per call. This pins the choice for later calls of this process (tests
 * cover both): 0 = choose per call, 128 or 256. INVALID_ARG for any other value. */
qp_status qp_select_linear_tile(int32_t token_rows);

/* How qp_linear would lay out a call (host arithmetic only, nothing is launched): token rows per workgroup tile,
 * workgroups per k chunk (including idle padding workgroups of the XCD mapping), k chunks (1 = not split) with
 * their 64-wide k-steps, and how much of the offered scratch the partial sums would take. Calls of at most 2 tokens
 * (decoding) run a kernel that streams the weights once instead, 4 weight rows per workgroup, never split:
 * token_rows_per_tile is then 1 or 2 (the tokens it computes) and workgroups = n / 4; a tiling pinned with
 * qp_select_linear_tile keeps such calls on the tiled kernel. */
typedef struct {
  int32_t token_rows_per_tile; /* 128 or 256; 1 or 2 for the weight-streaming kernel */
  int32_t workgroups;
  int32_t k_chunks;
  int32_t k_steps_per_chunk;   /* the last chunk may have fewer */
  size_t scratch_bytes;
} qp_linear_plan_info;
qp_status qp_linear_plan(int32_t m, int32_t n, int32_t k, size_t workspace_bytes, qp_linear_plan_info* out);

/* ---- the layer ------------------------------------------------------------------------------------------- */

/* Workspace of qp_layer_group / qp_layer_window_queries for groups of at most max_group_tokens tokens and a
 * window of n_window rows: the group's activations (h, q, k, v, attention output, x1, the MLP activation, the
 * rotary table, the scores), 32 MiB for split contractions, plus qp_workspace_bytes(layout, max_group_tokens,
 * n_window). 0 on bad arguments. */
size_t qp_layer_workspace_bytes(const qp_layout* layout, const qp_layer_shape* shape, int32_t max_group_tokens,
                                int32_t n_window);

/* One group through one layer.
 *   x_g [n_group_tokens][d_model] (read), x_out [n_group_tokens][d_model] (written; may alias x_g)
 *   pos / axis_stride: the group's position indices, as in qp_rope_table
 *   q_win [n_window][H_q][128]: this layer's scoring queries (qp_layer_window_queries), WINDOW rules only
 *   keep, group_token_base, cache, kept_idx_or_null: as in qp_topk_compact; the cache is this layer's
 * Scoring, top-k and compaction depend on the group's K and V only; they are enqueued on a library-owned side
 * stream (one per device, default priority, the one qp_prefill_video uses) forked from hip_stream after the QKV
 * projection and joined back into it before the call returns, so they run beside the attention and the
 * projections. Calls from several host threads are serialised while they enqueue.
 * Errors: INVALID_ARG, UNSUPPORTED (shape), CAPACITY (cache or workspace too small); on any error nothing is
 * launched and the cache is untouched. */
qp_status qp_layer_group(const qp_layout* layout, const qp_layer_shape* shape, const qp_layer_weights* weights,
                         const void* x_g, const int32_t* pos, int64_t axis_stride, int32_t n_group_tokens,
                         int32_t group_token_base, const void* q_win, int32_t n_window, qp_score_rule rule,
                         int32_t keep, qp_cache* cache, void* x_out, int32_t* kept_idx_or_null, void* workspace,
                         size_t workspace_bytes, void* hip_stream);

/* The text window's scoring queries of a layer from its hidden states: RMSNorm, W_q, b_q, rotary embedding.
 *   x_win [n_window][d_model], pos / axis_stride as above, q_win_out [n_window][H_q][128]. */
qp_status qp_layer_window_queries(const qp_layout* layout, const qp_layer_shape* shape,
                                  const qp_layer_weights* weights, const void* x_win, const int32_t* pos,
                                  int64_t axis_stride, int32_t n_window, void* q_win_out, void* workspace,
                                  size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* QP_LAYER_H_ */
