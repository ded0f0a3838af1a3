/*
 * qp.h -- C ABI of the QuickPrefill hot path for AMD MI355X (gfx950).
 *
 * QuickPrefill (Sec. 3.2 of the QuickVideo paper) prefills the video tokens of one
 * transformer layer group by group of frames. For each group:
 *   1. the group's queries attend to the pruned KV cache kept from earlier groups plus
 *      the group's own keys/values under a causal mask        -> qp_group_attend
 *   2. every new KV entry gets an importance score per KV head (Key Norms (small),
 *      Value Norms or Attention Scores, listed under Eq. 2)   -> qp_score_kv
 *   3. TopK keeps k = ceil(rho * N_g) entries per head and the survivors
 *      K_g[I_g], V_g[I_g] (Eq. 2) are appended to the cache   -> qp_topk_compact
 * qp_prefill_video runs the three steps over all groups of a layer.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer (HIP global memory) unless it says "host".
 *     All tensors are dense, row-major, 16-byte aligned. The qp_layout / qp_cache
 *     structs themselves live in HOST memory.
 *   - Tokens are the slow axis: activations are [tokens][heads][head_dim]. Query head qh
 *     reads KV head qh / (n_q_heads / n_kv_heads) (grouped-query attention).
 *   - The library allocates nothing and keeps no pointer after a call returns; scratch
 *     memory is the caller's `workspace` (size from qp_workspace_bytes, 256-byte aligned).
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the
 *     default stream), or ordered with respect to it (see qp_prefill_video). No call
 *     synchronises with the host or reads anything back: `cache->len` is host arithmetic and is already updated when a call returns, while
 *     the copies it describes may still be in flight on the stream.
 *   - Errors are returned as qp_status; nothing throws or aborts. Argument errors are
 *     detected on the host before anything is launched and leave `cache` untouched.
 *   - Same inputs give bit-identical kept indices, positions and cache contents.
 *   - Supported: dtype f32 or bf16, head_dim 64 or 128, n_q_heads a multiple of
 *     n_kv_heads, group size <= QP_MAX_GROUP_TOKENS.
 */
#ifndef QP_H_
#define QP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QP_MAX_GROUP_TOKENS 32768

typedef enum {
  QP_OK = 0,
  QP_ERR_INVALID_ARG = 1, /* NULL / misaligned pointer, non-positive size, bad enum          */
  QP_ERR_UNSUPPORTED = 2, /* dtype / head_dim / group size this build has no kernel for      */
  QP_ERR_CAPACITY = 3,    /* cache capacity or workspace too small                           */
  QP_ERR_HIP = 4,         /* a launch failed; qp_last_hip_error() holds the hipError_t value */
  /* not errors: returned by the consumer-side calls of qp_feed.h only */
  QP_FEED_END = 100,      /* the feed is closed and every published group has been taken     */
  QP_FEED_TIMEOUT = 101   /* nothing was published within the time-out                       */
} qp_status;

typedef enum { QP_F32 = 0, QP_BF16 = 1 } qp_dtype;

/* Element format of the pruned cache's K~ and V~. Sec. 3.2 prunes the cache to cut its memory; its bytes are
 * 2 * L * tokens * n_h * d_h * bytes-per-element (the KV-cache memory equation of App. D.2). QP_CACHE_FP8_E4M3
 * halves the last factor against bf16: kept rows are rounded to the 8-bit E4M3 format (OCP 8-bit floating point:
 * 4 exponent bits with bias 7, 3 mantissa bits, no infinities, largest value 448; nearest, ties to even, values
 * beyond +-448 saturate, NaN stays NaN) when qp_topk_compact stores them, and qp_group_attend widens them exactly
 * when it reads them. The group's own K, V (attended to before pruning) and the scores are unaffected.
 * Supported with bf16 layouts of head_dim 128. */
typedef enum { QP_CACHE_SAME = 0, QP_CACHE_FP8_E4M3 = 1 } qp_cache_format;

/* The three importance functions listed under Eq. 2 (Sec. 3.2). Larger score = kept first. */
typedef enum {
  QP_SCORE_KEY_NORM_SMALL = 0, /* s = -||K_g[j,h,:]||_2  (the paper's default)                  */
  QP_SCORE_VALUE_NORM = 1,     /* s = +||V_g[j,h,:]||_2                                          */
  QP_SCORE_WINDOW_ATTN = 2,    /* "Attention Scores": softmax attention mass that key j of KV
                                  head h receives from the text-query window, softmax taken over
                                  the group's own keys, summed over the window's queries and over
                                  the query heads that map to h                                  */
  QP_SCORE_WINDOW_LOGIT = 3,   /* variant of the above without the softmax (the literal
                                  s = matmul(K_g, Q) of the list): scale * sum of the logits
                                  q.k over the same queries and heads = one dot product per key  */
  QP_SCORE_SHARED_HEADS = 0x100 /* flag, OR-ed into a rule above: head-shared selection. Every KV
                                  head's score of a token becomes the sum of all heads' scores
                                  (f32, in head order), so the per-head TopK of Eq. 2 -- which
                                  writes one index set I_g -- keeps the same tokens for all heads */
} qp_score_rule;

/* Which attention kernel qp_group_attend uses. AUTO picks the MFMA kernel when the
 * layout allows it (bf16, head_dim 128), else the scalar one. */
typedef enum {
  QP_ATTEND_AUTO = 0,
  QP_ATTEND_SCALAR = 1,
  QP_ATTEND_MFMA = 2,
  QP_ATTEND_MFMA_DECODE = 3 /* reported by qp_attend_plan only: AUTO's kernel for at most 32 stacked rows
                               per KV head (decode-shaped calls); not selectable */
} qp_attend_kernel;

typedef struct {
  int32_t n_q_heads;   /* H_q                                                   */
  int32_t n_kv_heads;  /* H_kv, divides H_q                                     */
  int32_t head_dim;    /* d                                                     */
  int32_t dtype;       /* qp_dtype of q/k/v/out and of the cache                */
  float softmax_scale; /* logit scale; 0 means 1/sqrt(head_dim)                 */
} qp_layout;

/* The pruned KV cache of one layer (Sec. 3.2, "store the corresponding KV cache"):
 * the same number of entries `len` for every KV head, in ascending token order. */
typedef struct {
  void* k;          /* device, [n_kv_heads][capacity][head_dim], layout dtype (or 1 byte per element, see format) */
  void* v;          /* device, [n_kv_heads][capacity][head_dim]                          */
  int32_t* pos;     /* device, [n_kv_heads][capacity]: video-token index of each entry   */
  int32_t capacity; /* entries per head the buffers can hold                             */
  int32_t len;      /* host: entries per head currently valid; updated by qp_topk_compact */
  int32_t format;   /* qp_cache_format of k and v; 0 (QP_CACHE_SAME) = the layout's dtype */
} qp_cache;

/* ---- host arithmetic (no device work) ------------------------------------------------ */

/* k of Eq. 2 for a group of n tokens: ceil(retention * n - 1e-9) clamped to [1, n]; 0 if n <= 0.
 * retention outside (0, 1] returns -1. */
int64_t qp_keep_count(int64_t n_group_tokens, double retention);

/* Entries per head the cache must hold after all frame-aligned groups of a video
 * (groups of group_frames frames, the last one possibly shorter). -1 on bad arguments. */
int64_t qp_cache_capacity(int32_t n_frames, int32_t tokens_per_frame, int32_t group_frames, double retention);

/* The frame-aligned groups of a video (Sec. 3.2, "Group-Based Prefill": groups of about N_g tokens; Tables 1-2 give
 * the size in frames): group i covers tokens [first_token[i], first_token[i] + n_tokens[i]); every group has
 * group_frames frames except possibly the last. Returns the number of groups G; writes the first
 * min(G, max_groups) entries of each HOST array that is not NULL. -1 on bad arguments. */
int32_t qp_group_bounds(int32_t n_frames, int32_t tokens_per_frame, int32_t group_frames, int32_t* first_token,
                        int32_t* n_tokens, int32_t max_groups);

/* The conversions of the 8-bit cache format (qp_cache_format) on the host, bit patterns in and out: the E4M3 code
 * of a bf16 value (nearest, ties to even, saturating at +-448, NaN to the NaN code 0x7f | sign) -- the same routine
 * the compaction kernel runs -- and a code's value as bf16 (exact). */
uint8_t qp_e4m3_from_bf16(uint16_t bf16_bits);
uint16_t qp_bf16_from_e4m3(uint8_t code);

/* Bytes of workspace that every entry point accepts for groups of at most max_group_tokens
 * tokens and a query window of n_window rows (includes 2 x 128 MiB of key-split scratch for the
 * attention launches of qp_prefill_video). 0 on bad arguments. */
size_t qp_workspace_bytes(const qp_layout* layout, int32_t max_group_tokens, int32_t n_window);

/* ---- the hot path ----------------------------------------------------------------------- */

/* Group attention (Sec. 2.1 softmax self-attention, applied per group as in Sec. 3.2).
 *   q_g [n_group_tokens][H_q][d], k_g, v_g [n_group_tokens][H_kv][d]  (read)
 *   cache: entries [0, cache->len) of every head are read; may be NULL or len 0 (first group)
 *   out_g [n_group_tokens][H_q][d], layout dtype (written)
 *   lse_or_null [H_q][n_group_tokens] f32: natural-log sum of exp(scale*q.k) over the visible
 *     keys of each row (written if not NULL)
 * Row i of query head qh sees all cache entries of KV head qh/R and group tokens j <= i.
 * Arithmetic: products and sums in f32 (bf16 inputs are widened exactly; the MFMA kernel
 * rounds the softmax numerators to bf16 before the P.V product); output rounded to nearest even.
 * The same call serves the stages that follow video prefill (Sec. 2.1: text-token prefill, then
 * decoding): a text chunk or a single new token is a "group" of n_group_tokens >= 1 rows attending
 * to the whole pruned cache plus itself.
 *   workspace: optional device scratch (256-byte aligned), may be NULL. When a launch would have too
 *     few rows to fill the GPU against a long cache, the cache is dealt to key chunks whose partial
 *     results a second launch merges; the partials ([chunks][rows][d+1] f32, as many chunks as fit)
 *     live in this scratch. Two kernels do this: calls of at most 32 stacked rows per KV head
 *     (n_group_tokens * H_q/H_kv <= 32: decoding) run a kernel in which every wavefront streams its
 *     own blocks of keys; larger ones split the tiles of the large kernel (at most 128 chunks).
 *     Launches of several rounds of workgroups use the scratch too: the row blocks of a partly
 *     filled last round (the group's earliest tokens) are split over up to 8 key chunks, so that
 *     their chunks fill the compute units evenly (partials for those rows only).
 *     Without scratch nothing is split. Calls that may overlap on different streams need distinct
 *     scratch. qp_attend_plan reports the choice.
 * Errors: INVALID_ARG (NULL/misaligned pointers, n_group_tokens <= 0, bad layout),
 * UNSUPPORTED (dtype/head_dim/group size). The cache is not modified. */
qp_status qp_group_attend(const qp_layout* layout, const void* q_g, const void* k_g, const void* v_g,
                          int32_t n_group_tokens, const qp_cache* cache, void* out_g, float* lse_or_null,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* qp_group_attend for callers that cannot allocate or hand over scratch memory: code under HIP graph capture,
 * tight serving loops (one decode step or one text chunk per call), harnesses that forbid hipMalloc. Same
 * arguments and results as qp_group_attend without the workspace pair: the key split's partial results live in a
 * device array of QP_NOALLOC_SCRATCH_BYTES that the library holds on every GPU it runs on until the process ends.
 * The call allocates nothing and frees nothing. With a workspace of exactly QP_NOALLOC_SCRATCH_BYTES,
 * qp_group_attend takes the same launch layout and returns the same bits.
 *   Limit: n_group_tokens * H_q <= QP_NOALLOC_MAX_ROWS (decode steps and text chunks; a chunk of that many rows
 *     leaves room for at least 8 key chunks), else QP_ERR_CAPACITY and nothing is launched.
 *   The array keeps the previous call's contents; nothing in it needs clearing (every partial result is written
 *     before the merge reads it). All calls on one GPU share the array: calls that may overlap on one GPU
 *     (different streams, different host threads) race -- use qp_group_attend with distinct workspaces for those.
 *   Other errors as qp_group_attend; QP_ERR_HIP if the array's device address cannot be obtained. */
#define QP_NOALLOC_SCRATCH_BYTES (8u << 20)
#define QP_NOALLOC_MAX_ROWS 2048
qp_status qp_group_attend_noalloc(const qp_layout* layout, const void* q_g, const void* k_g, const void* v_g,
                                  int32_t n_group_tokens, const qp_cache* cache, void* out_g, float* lse_or_null,
                                  void* hip_stream);

/* Importance scores of a group's new KV entries (the functions listed under Eq. 2).
 *   k_g, v_g as above (the norm rules read only the tensor they name; the other may be NULL)
 *   q_win [n_window][H_q][d]: the text-query window (the two WINDOW rules only, else ignored)
 *   scores [H_kv][n_group_tokens] f32 (written)
 * f32 arithmetic. Errors as above; a WINDOW rule with q_win NULL or n_window <= 0 is INVALID_ARG;
 * CAPACITY if the workspace is too small (the WINDOW rules need qp_workspace_bytes(layout,
 * n_group_tokens, n_window)). */
qp_status qp_score_kv(const qp_layout* layout, qp_score_rule rule, const void* k_g, const void* v_g,
                      int32_t n_group_tokens, const void* q_win, int32_t n_window, float* scores,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* TopK of Eq. 2 per KV head and compaction of the survivors into the cache.
 *   scores [H_kv][n_group_tokens] f32 (read). Ordering: larger first, equal scores (and
 *     -0.0 == +0.0) by lower token index; scores must not be NaN.
 *   keep: k, 1 <= keep <= n_group_tokens
 *   group_token_base: video-token index of the group's first token (recorded in cache->pos)
 *   cache: rows K_g[I], V_g[I] are appended at [len, len+keep) of every head in ascending
 *     token order, pos gets group_token_base + I, then cache->len += keep (host side)
 *   kept_idx_or_null [H_kv][keep] int32: group-local kept indices, ascending (written if not NULL)
 *   workspace, workspace_bytes: not used (selection and copy are one launch); may be NULL / 0
 * Errors: INVALID_ARG, UNSUPPORTED, CAPACITY (len + keep > capacity); on any error the cache is untouched. */
qp_status qp_topk_compact(const qp_layout* layout, const float* scores, const void* k_g, const void* v_g,
                          int32_t n_group_tokens, int32_t keep, int32_t group_token_base, qp_cache* cache,
                          int32_t* kept_idx_or_null, void* workspace, size_t workspace_bytes, void* hip_stream);

/* One layer of QuickPrefill over a whole video (Sec. 3.2): frame-aligned groups of
 * group_frames frames in order, each attended, scored, pruned and compacted.
 *   q [N][H_q][d], k, v [N][H_kv][d] with N = n_frames * tokens_per_frame
 *   q_win [n_window][H_q][d] or NULL (needed by QP_SCORE_WINDOW_ATTN)
 *   cache: appended starting at cache->len (normally 0); entries already in it are visible
 *     to every group. Needs capacity >= len + qp_cache_capacity(...).
 *   out [N][H_q][d]
 * All arguments are validated before the first launch. Scoring and compaction of a group do not
 * depend on its attention, and the attention of group g+1 depends on the compaction of group g but
 * not on the attention of group g; the call uses two library-owned streams per device (created on
 * first use on the current device, default priority) for the scoring/compaction chain and for every
 * other group's attention (the latter only when a group's attention launch is under two rounds of
 * workgroups; larger launches all run on hip_stream). They are forked from hip_stream at entry and joined back into it before
 * the call returns: work the caller enqueues on hip_stream afterwards is ordered after all of this
 * call's work. The call only enqueues (it never waits for the GPU); calls from several host threads
 * are serialised while they enqueue, because they share those streams.
 * Failure after the first launch (QP_ERR_HIP from a launch or a stream call): nothing further is enqueued, the
 * library's streams are still joined back into hip_stream, the groups already enqueued run to completion, and
 * cache->len is restored to its value at entry (rows beyond it, and `out`, then hold unspecified data). */
qp_status qp_prefill_video(const qp_layout* layout, int32_t n_frames, int32_t tokens_per_frame,
                           int32_t group_frames, double retention, qp_score_rule rule, const void* q,
                           const void* k, const void* v, const void* q_win, int32_t n_window, qp_cache* cache,
                           void* out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- control / diagnostics ------------------------------------------------------------------ */

/* How qp_group_attend would lay out a call (host arithmetic only, nothing is launched): which kernel,
 * how many workgroups, whether the cache is split over key chunks (key_chunks > 1: two launches, the
 * second merges the chunks' partial results; tiles_per_chunk counts 64-key cache tiles) and for how many
 * row blocks of 256 stacked rows per KV head (split_row_blocks: all of them when few rows meet a long
 * cache; only those of the launch's last, partly filled round of workgroups when there are several
 * rounds, so that their chunks fill the compute units evenly), whether rows are dealt to workgroups as
 * mirrored early/late half blocks (launches of at most one workgroup per compute unit) or consecutively,
 * and how much of the offered workspace the split would use.
 * For the scalar kernel only `kernel` and key_chunks = 1 are meaningful. */
typedef struct {
  int32_t kernel;          /* QP_ATTEND_SCALAR, QP_ATTEND_MFMA or QP_ATTEND_MFMA_DECODE */
  int32_t workgroups;      /* of the first launch, all chunks and idle padding workgroups included */
  int32_t key_chunks;
  int32_t tiles_per_chunk; /* 0 when key_chunks == 1 */
  int32_t mirrored_rows;
  size_t scratch_bytes;
  int32_t split_row_blocks; /* 0 when key_chunks == 1 (MFMA kernel; the decode kernel splits all of its rows) */
} qp_attend_plan_info;
qp_status qp_attend_plan(const qp_layout* layout, int32_t n_group_tokens, int32_t cache_len,
                         size_t workspace_bytes, qp_attend_plan_info* out);


/* Choose the attention kernel for later qp_group_attend / qp_prefill_video calls of this
 * process (tests use it to cover both). Returns INVALID_ARG for an unknown value. */
qp_status qp_select_attend_kernel(int32_t which);

/* Test seam for the error paths: the n_checks-th launch check from now on (every entry point of this header checks
 * once after it has enqueued its launches; qp_prefill_video checks three times per group) reports QP_ERR_HIP with
 * hipErrorLaunchFailure although the GPU work was enqueued and runs normally. 0 switches it off. Process-wide. */
qp_status qp_debug_fail_after(int32_t n_checks);

const char* qp_status_string(qp_status s); /* static string, never NULL */
int qp_last_hip_error(void);               /* hipError_t of the last failed launch on this thread, 0 if none */
const char* qp_version(void);              /* static string */

#ifdef __cplusplus
}
#endif
#endif /* QP_H_ */
