"""fp64 CPU oracle for the QuickPrefill path (group prefill + KV-cache pruning).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. Only the tests, the smoke check and
the benchmark's CPU-baseline leg may import it. It shares no code with the HIP
library, imports nothing from the GPU package, and is deliberately plain: every
function is the paper's definition written out with numpy in float64, one group
/ one head at a time, with a BLAS matmul as the only library step. No tiling,
no online softmax, no fusion.

What the paper fixes (Sec. 3.2 "Group-Based Prefill", "Group-Based KV Cache
Pruning", Eq. 2 and the three score functions listed under it) and what it
leaves open is resolved as follows; each reading is also listed in the design
notes of the repository:

  * A group's queries see the *pruned* KV kept from all earlier groups (fully
    visible) plus the group's own, un-pruned KV under a causal mask; the group is
    pruned after its own attention (Sec. 3.2 says pruning happens "when
    processing each group"; Sec. 4.2 says rho = 0.5 halves the computation).
  * Groups are frame-aligned: g frames each, the last one possibly shorter
    (Tables 1-2 give group size in frames).
  * k = ceil(rho * N_g) per group, from the actual group length, clamped to
    [1, N_g]; a 1e-9 guard keeps products such as 0.07*100 = 7.000000000000001
    from rounding up (Eq. 2 gives k = rho * N_g with no rounding rule).
  * One index set per KV head (the L2 norm over head_dim of a
    [tokens, heads, head_dim] tensor leaves a head axis); same k for all heads.
  * Key Norms (small): s = -||K_g[j,h,:]||_2. Value Norms: s = +||V_g[j,h,:]||_2.
  * Attention Scores: s = matmul(K_g, Q) is read as the attention mass a key
    receives from the text-query window: softmax over the group's own N_g keys of
    scale * q.k for every window query of every query head that maps to the KV
    head, summed over those queries and heads. No mask (text follows video).
  * TopK ties go to the lower token index; survivors are stored in ascending
    token order.
  * scale = 1/sqrt(head_dim) unless given.

Parity status: every function below is pinned by the CPU tests (brute force on
tiny inputs, library softmax / scaled-dot-product attention, closed forms, the
paper's printed memory figures, hand-computed top-k examples, invariants). The
whole path against numbers printed in the paper: parity unpinned -- the paper
prints no intermediate or output of this path.
"""
from __future__ import annotations

import math

import numpy as np

RULES = ("key_norm_small", "value_norm", "window_attn")


# --------------------------------------------------------------------------- #
# Eq. 2: k = rho * N_g
# --------------------------------------------------------------------------- #
def keep_count(n_group_tokens: int, retention: float) -> int:
    """Number of KV entries a group of n tokens keeps per head (Eq. 2, k = rho*N_g, rounded up)."""
    if n_group_tokens <= 0:
        return 0
    k = int(math.ceil(retention * n_group_tokens - 1e-9))
    return max(1, min(n_group_tokens, k))


def group_bounds(n_frames: int, tokens_per_frame: int, group_frames: int):
    """Frame-aligned partition of the video tokens into G groups (Sec. 3.2, Group-Based Prefill)."""
    out = []
    f = 0
    while f < n_frames:
        g = min(group_frames, n_frames - f)
        out.append((f * tokens_per_frame, g * tokens_per_frame))
        f += g
    return out


def final_cache_len(n_frames, tokens_per_frame, group_frames, retention) -> int:
    return sum(keep_count(n, retention) for _, n in group_bounds(n_frames, tokens_per_frame, group_frames))


# --------------------------------------------------------------------------- #
# Group attention (Sec. 2.1: softmax self-attention; Sec. 3.2: per group)
# --------------------------------------------------------------------------- #
def attend_group(q_g, k_g, v_g, cache_k, cache_v, scale=None, rows=None, return_lse=False):
    """Attention output of one group.

    q_g [N_g, H_q, d]; k_g, v_g [N_g, H_kv, d]; cache_k, cache_v [H_kv, C, d] (C may be 0).
    Query token i of head qh (KV head qh // R) sees all C cache entries and group
    tokens j <= i. rows: optional list of group-token indices to evaluate (others
    are skipped; the result then has len(rows) rows).
    Returns O [n_rows, H_q, d] (and lse [H_q, n_rows], natural log, if asked).
    """
    q_g = np.asarray(q_g, dtype=np.float64)
    k_g = np.asarray(k_g, dtype=np.float64)
    v_g = np.asarray(v_g, dtype=np.float64)
    n_g, h_q, d = q_g.shape
    h_kv = k_g.shape[1]
    r = h_q // h_kv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    c = 0 if cache_k is None else cache_k.shape[1]
    row_idx = np.arange(n_g) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.zeros((len(row_idx), h_q, d), dtype=np.float64)
    lse = np.zeros((h_q, len(row_idx)), dtype=np.float64)
    col = np.arange(n_g)
    for qh in range(h_q):
        h = qh // r
        if c > 0:
            keys = np.concatenate([np.asarray(cache_k[h], dtype=np.float64), k_g[:, h, :]], axis=0)
            vals = np.concatenate([np.asarray(cache_v[h], dtype=np.float64), v_g[:, h, :]], axis=0)
        else:
            keys, vals = k_g[:, h, :], v_g[:, h, :]
        logits = scale * (q_g[row_idx, qh, :] @ keys.T)                  # [n_rows, C + N_g]
        visible = np.ones_like(logits, dtype=bool)
        visible[:, c:] = col[None, :] <= row_idx[:, None]                # causal inside the group
        logits = np.where(visible, logits, -np.inf)
        m = logits.max(axis=1, keepdims=True)
        p = np.exp(logits - m)
        z = p.sum(axis=1, keepdims=True)
        out[:, qh, :] = (p / z) @ vals
        lse[qh] = (m + np.log(z))[:, 0]
    return (out, lse) if return_lse else out


# --------------------------------------------------------------------------- #
# Importance scores (the three functions listed under Eq. 2)
# --------------------------------------------------------------------------- #
def score_kv(rule, k_g, v_g, q_win=None, scale=None):
    """s [H_kv, N_g] for one group; larger = more important. A rule name ending in "+shared" is that rule followed by
    share_scores_across_heads (head-shared selection)."""
    if rule.endswith("+shared"):
        return share_scores_across_heads(score_kv(rule[:-len("+shared")], k_g, v_g, q_win, scale))
    k_g = np.asarray(k_g, dtype=np.float64)
    n_g, h_kv, d = k_g.shape
    if rule == "key_norm_small":
        return -np.sqrt((k_g * k_g).sum(axis=2)).T.copy()
    if rule == "value_norm":
        v_g = np.asarray(v_g, dtype=np.float64)
        return np.sqrt((v_g * v_g).sum(axis=2)).T.copy()
    if rule == "window_attn":
        q_win = np.asarray(q_win, dtype=np.float64)
        w, h_q, _ = q_win.shape
        r = h_q // h_kv
        if scale is None:
            scale = 1.0 / math.sqrt(d)
        s = np.zeros((h_kv, n_g), dtype=np.float64)
        for qh in range(h_q):
            h = qh // r
            logits = scale * (q_win[:, qh, :] @ k_g[:, h, :].T)          # [W, N_g]
            p = np.exp(logits - logits.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            s[h] += p.sum(axis=0)
        return s
    if rule == "window_logit":
        # Variant of the attention-score rule without the softmax: the literal `s = matmul(K_g, Q)` of the list under
        # Eq. 2, i.e. the scaled logits summed over the window's queries and the query heads of the KV head.
        q_win = np.asarray(q_win, dtype=np.float64)
        w, h_q, _ = q_win.shape
        r = h_q // h_kv
        if scale is None:
            scale = 1.0 / math.sqrt(d)
        s = np.zeros((h_kv, n_g), dtype=np.float64)
        for qh in range(h_q):
            logits = scale * (q_win[:, qh, :] @ k_g[:, qh // r, :].T)    # [W, N_g]
            s[qh // r] += logits.sum(axis=0)
        return s
    raise ValueError(f"unknown scoring rule {rule!r}")


def share_scores_across_heads(scores):
    """Head-shared selection (Eq. 2 writes one index set I_g without a head index): every KV head scores a token by
    the sum of all heads' scores, so the per-head TopK returns the same set for every head."""
    scores = np.asarray(scores, dtype=np.float64)
    total = np.zeros(scores.shape[1], dtype=np.float64)
    for h in range(scores.shape[0]):       # in head order
        total = total + scores[h]
    return np.broadcast_to(total, scores.shape).copy()


# --------------------------------------------------------------------------- #
# TopK of Eq. 2
# --------------------------------------------------------------------------- #
def topk_select(scores, k):
    """Indices [H, k] of the k largest scores per head; ties -> lower index; ascending order."""
    scores = np.asarray(scores)
    h, n = scores.shape
    out = np.zeros((h, k), dtype=np.int64)
    for i in range(h):
        order = sorted(range(n), key=lambda j: (-scores[i, j], j)) if n <= 64 else \
            np.lexsort((np.arange(n), -scores[i]))
        out[i] = np.sort(np.asarray(order[:k], dtype=np.int64))
    return out


# --------------------------------------------------------------------------- #
# Variant: the pruned cache kept in 8 bits per element
# --------------------------------------------------------------------------- #
def fp8_e4m3_round(x):
    """Nearest value of the 8-bit E4M3 floating-point format, returned as float64.

    The format (OCP 8-bit floating point, E4M3): 1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits, no
    infinities; normal values (1 + m/8) * 2^e for e in [-6, 8] (the largest, 1.75 * 2^8 = 448, because the code above
    it is NaN), subnormal values (m/8) * 2^-6. Rounding is to nearest, ties to the even mantissa; magnitudes that
    would round above 448 saturate to +-448 (a reading: the format also allows NaN there); NaN stays NaN.
    """
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    _, ex = np.frexp(a)                              # a = f * 2^ex, f in [0.5, 1): exponent of the leading bit is ex - 1
    e = np.maximum(ex - 1, -6)                       # subnormals share the smallest normal exponent
    quantum = np.ldexp(1.0, e - 3)                   # spacing of representable values in that binade
    r = np.rint(a / quantum) * quantum               # np.rint rounds half to even; both operations are exact in float64
    r = np.minimum(r, 448.0)
    r = np.where(np.isnan(x), np.nan, r)
    return np.copysign(r, x)


CACHE_FORMATS = (None, "fp8_e4m3")


def _store_cache_rows(rows, cache_format):
    """Rows as the cache holds them: unchanged, or rounded to the cache's element format."""
    if cache_format is None:
        return rows
    if cache_format == "fp8_e4m3":
        return fp8_e4m3_round(rows)
    raise ValueError(f"unknown cache format {cache_format!r}")


# --------------------------------------------------------------------------- #
# The whole path for one layer
# --------------------------------------------------------------------------- #
def select_all_groups(k, v, q_win, n_frames, tokens_per_frame, group_frames, retention, rule, scale=None):
    """Kept indices of every group: [(base, n_g, idx[H_kv, k_g] group-local, scores[H_kv, n_g])].

    Scores depend only on the group's own K/V and the window queries (Eq. 2 writes
    s(K_g, V_g)), so this needs no attention.
    """
    out = []
    for base, n_g in group_bounds(n_frames, tokens_per_frame, group_frames):
        s = score_kv(rule, k[base:base + n_g], v[base:base + n_g], q_win, scale)
        idx = topk_select(s, keep_count(n_g, retention))
        out.append((base, n_g, idx, s))
    return out


def gather_cache(k, v, selections, upto_group, cache_format=None):
    """Cache contents before group `upto_group`: K~ [H_kv, C, d], V~ [H_kv, C, d], pos [H_kv, C]. With a cache_format
    the kept rows are rounded to it when they enter the cache (what later groups attend to)."""
    k = np.asarray(k)
    h_kv, d = k.shape[1], k.shape[2]
    ks, vs, ps = [], [], []
    for base, n_g, idx, _ in selections[:upto_group]:
        pos = base + idx                                                   # [H_kv, k_g] global token index
        ks.append(_store_cache_rows(np.stack([k[pos[h], h, :] for h in range(h_kv)]), cache_format))
        vs.append(_store_cache_rows(np.stack([v[pos[h], h, :] for h in range(h_kv)]), cache_format))
        ps.append(pos)
    if not ks:
        return (np.zeros((h_kv, 0, d)), np.zeros((h_kv, 0, d)), np.zeros((h_kv, 0), dtype=np.int64))
    return np.concatenate(ks, axis=1), np.concatenate(vs, axis=1), np.concatenate(ps, axis=1)


def prefill_video(q, k, v, q_win, n_frames, tokens_per_frame, group_frames, retention, rule, scale=None,
                  cache_format=None):
    """One layer of QuickPrefill, group by group, in the order the method states. cache_format: element format of
    the pruned cache (None: the inputs' own; "fp8_e4m3": kept rows are rounded to 8 bits when they are stored; the
    group's own K, V, which it attends to before pruning, and the scores are not affected).

    Returns O [N, H_q, d], cache K~ [H_kv, C_G, d], V~ [H_kv, C_G, d], pos [H_kv, C_G],
    and the per-group selections.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    n, h_q, d = q.shape
    h_kv = k.shape[1]
    out = np.zeros((n, h_q, d), dtype=np.float64)
    cache_k = np.zeros((h_kv, 0, d))
    cache_v = np.zeros((h_kv, 0, d))
    cache_pos = np.zeros((h_kv, 0), dtype=np.int64)
    selections = []
    for base, n_g in group_bounds(n_frames, tokens_per_frame, group_frames):
        sl = slice(base, base + n_g)
        # 1. the group attends to the pruned cache so far + itself (causal)
        out[sl] = attend_group(q[sl], k[sl], v[sl], cache_k, cache_v, scale)
        # 2. score the group's new KV entries per KV head
        s = score_kv(rule, k[sl], v[sl], q_win, scale)
        # 3. TopK (Eq. 2)
        idx = topk_select(s, keep_count(n_g, retention))
        # 4. K~_g = K_g[I_g], V~_g = V_g[I_g] appended to the cache
        pos = base + idx
        cache_k = np.concatenate([cache_k, _store_cache_rows(np.stack([k[pos[h], h, :] for h in range(h_kv)]),
                                                             cache_format)], axis=1)
        cache_v = np.concatenate([cache_v, _store_cache_rows(np.stack([v[pos[h], h, :] for h in range(h_kv)]),
                                                             cache_format)], axis=1)
        cache_pos = np.concatenate([cache_pos, pos], axis=1)
        selections.append((base, n_g, idx, s))
    return out, cache_k, cache_v, cache_pos, selections


# --------------------------------------------------------------------------- #
# Memory models (Appendix D: activation-memory and KV-cache-memory equations)
# --------------------------------------------------------------------------- #
def attn_activation_bytes(batch, seq, n_heads, d_head, b_r, b_c, elem_bytes=2):
    """Appendix D.1, attention block: Q, K, V plus one B_r x B_c block of the attention matrix."""
    return (3 * batch * seq * n_heads * d_head + batch * n_heads * b_r * b_c) * elem_bytes


def mlp_activation_bytes(batch, seq, d_model, d_ff, elem_bytes=2):
    """Appendix D.1, SwiGLU MLP block."""
    return batch * seq * (2 * d_model + 4 * d_ff) * elem_bytes


def kv_cache_bytes(n_layers, n_tokens, n_heads, d_head, elem_bytes=2, retention=1.0):
    """Appendix D.2: 2 * L * tokens * n_h * d_h * bytes; Sec. 3.2: pruning divides it by 1/rho."""
    return 2 * n_layers * n_tokens * n_heads * d_head * elem_bytes * retention
