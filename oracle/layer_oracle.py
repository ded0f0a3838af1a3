"""fp64 CPU oracle for one decoder layer around the QuickPrefill path, one group at a time.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import it. It shares no code with the HIP library and imports nothing from the GPU
package. Every function is the textbook definition written out with numpy in float64; the only library
step is a BLAS matmul.

What it covers. Sec. 3.2 of the paper prefills a video group by group so that the activations of a
transformer block exist for one group at a time (Appendix D.1 prices the two blocks: attention with
Q, K, V of the group, and the SwiGLU MLP, whose definition the appendix prints:
SwiGLU(x) = W_down (SiLU(W_gate x) * W_up x), SiLU(x) = x * sigmoid(x)). The block modelled here is the
pre-norm decoder layer of the Qwen2.5 family the paper evaluates:

    h   = RMSNorm(x; w_ln1)                         y_i = x_i / sqrt(mean(x^2) + eps) * w_i
    q,k,v = h W_q^T + b_q, h W_k^T + b_k, h W_v^T + b_v     (heads split token-major: [N, H, d])
    q,k = RoPE(q), RoPE(k)                          multimodal rotary embedding, see mrope_cos_sin
    a   = QuickPrefill group attention over (pruned cache of this layer, this group)   [qp_oracle.attend_group]
    cache update: score, top-k, gather               [qp_oracle.score_kv / topk_select]
    x1  = x + a W_o^T
    x2  = x1 + SwiGLU(RMSNorm(x1; w_ln2))

Readings (the paper does not describe the layer beyond Appendix D.1; these are stated in the design notes):
  * The rotary embedding is applied before the keys enter the cache, so cached keys carry their own
    positions and are never re-rotated.
  * Rotary convention: the head dimension is split in two halves; component i of the first half pairs with
    component i + d/2 of the second. Frequency i is theta^(-2i/d). Each token has three position
    indices (temporal, height, width); frequencies [0, s0) take the temporal index, [s0, s0+s1) the
    height, the rest the width (s0 + s1 + s2 = d/2). Equal indices on the three axes reduce this to the
    ordinary one-dimensional rotary embedding.
  * The scoring queries of the "attention scores" rule are the text window's queries of the same layer:
    its hidden states are an input of the layer (they come from the text side), projected and rotated
    with the layer's own W_q, b_q.
  * `store` is applied wherever the product keeps a tensor in its storage type (bf16) so that top-k
    decisions are taken on keys of the same precision on both sides; the default keeps float64 throughout.

Parity status: rms_norm, mrope_cos_sin / apply_rotary, silu / swiglu_mlp and linear are pinned by the CPU
tests (closed forms, the relative-position invariance of rotary embeddings, norm preservation, reduction to
the one-dimensional embedding, hand-computed small cases, library silu). window_queries / project_queries: a
one-token case worked by hand (tests/golden/hand_window_queries.txt), scale invariance (the norm is there), which
parameters they depend on, bias-before-rotation, and equality with layer_group's own q for the same tokens.
layer_group's wiring: the same block built from library routines only (torch rms_norm / linear / silu / scaled-dot-
product attention, rotation as a complex product), its composition from the pinned parts, perturbation pins on
every edge of the residual stream, identity with zero output projections. layer_stack: rho = 1 equals one group;
with rho < 1 every layer's kept set is the top-k of that layer's own keys under that layer's own window queries.
layer_group against numbers printed in the paper: parity unpinned -- the paper prints no activation of any layer.
"""
from __future__ import annotations

import numpy as np

from . import qp_oracle as qo


def bf16_round(x):
    """Round float64 values to the nearest bf16 (ties to even), returned as float64."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


def rms_norm(x, w, eps):
    """y[n, i] = x[n, i] / sqrt(mean_i x[n, i]^2 + eps) * w[i]."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(w, dtype=np.float64)


def linear(x, w, b=None):
    """y = x W^T + b with W stored [out, in]."""
    y = np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T
    if b is not None:
        y = y + np.asarray(b, dtype=np.float64)
    return y


def mrope_cos_sin(pos3, head_dim, theta, sections):
    """cos, sin [N, d/2] of the rotation angles: angle[n, i] = pos3[axis(i), n] * theta^(-2i/d)."""
    pos3 = np.asarray(pos3, dtype=np.float64)
    half = head_dim // 2
    assert pos3.shape[0] == 3 and sum(sections) == half
    axis = np.repeat(np.arange(3), sections)                       # which position index frequency i uses
    inv_freq = theta ** (-2.0 * np.arange(half) / head_dim)
    ang = pos3[axis, :].T * inv_freq[None, :]                      # [N, half]
    return np.cos(ang), np.sin(ang)


def apply_rotary(x, cos, sin):
    """x [N, H, d]: (x_i, x_{i+d/2}) -> (x_i cos - x_{i+d/2} sin, x_{i+d/2} cos + x_i sin)."""
    x = np.asarray(x, dtype=np.float64)
    half = x.shape[-1] // 2
    a, b = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x):
    x = np.asarray(x, dtype=np.float64)
    return x / (1.0 + np.exp(-x))


def swiglu_mlp(x, w_gate, w_up, w_down, store=lambda t: t):
    """Appendix D.1: W_down (SiLU(W_gate x) * W_up x)."""
    act = store(silu(linear(x, w_gate)) * linear(x, w_up))
    return linear(act, w_down)


def project_queries(h, w_q, b_q, pos3, shape, store=lambda t: t):
    """Rotated queries [N, H_q, d] of normalised hidden states h."""
    n = h.shape[0]
    cos, sin = mrope_cos_sin(pos3, shape["head_dim"], shape["rope_theta"], shape["mrope_section"])
    q = linear(h, w_q, b_q).reshape(n, shape["n_q_heads"], shape["head_dim"])
    return store(apply_rotary(q, cos, sin))


def window_queries(x_win, pos3_win, weights, shape, store=lambda t: t):
    """The text window's scoring queries of this layer, from its hidden states."""
    h = store(rms_norm(x_win, weights["ln1"], shape["rms_eps"]))
    return project_queries(h, weights["w_q"], weights["b_q"], pos3_win, shape, store)


def layer_group(x_g, pos3_g, weights, shape, cache_k, cache_v, q_win, rule, retention, store=lambda t: t):
    """One group through one layer. cache_k / cache_v: this layer's pruned cache [H_kv, C, d] so far.

    Returns x_out [N_g, d_model], the group's kept indices [H_kv, k] (group-local, ascending), the rows
    K~_g, V~_g [H_kv, k, d] to append to the cache, and a dict of intermediates.
    """
    x_g = np.asarray(x_g, dtype=np.float64)
    n_g = x_g.shape[0]
    h_q, h_kv, d = shape["n_q_heads"], shape["n_kv_heads"], shape["head_dim"]
    h = store(rms_norm(x_g, weights["ln1"], shape["rms_eps"]))
    cos, sin = mrope_cos_sin(pos3_g, d, shape["rope_theta"], shape["mrope_section"])
    q = store(apply_rotary(linear(h, weights["w_q"], weights["b_q"]).reshape(n_g, h_q, d), cos, sin))
    k = store(apply_rotary(linear(h, weights["w_k"], weights["b_k"]).reshape(n_g, h_kv, d), cos, sin))
    v = store(linear(h, weights["w_v"], weights["b_v"]).reshape(n_g, h_kv, d))
    a = store(qo.attend_group(q, k, v, cache_k, cache_v))
    s = qo.score_kv(rule, k, v, q_win)
    idx = qo.topk_select(s, qo.keep_count(n_g, retention))
    new_k = np.stack([k[idx[j], j, :] for j in range(h_kv)])
    new_v = np.stack([v[idx[j], j, :] for j in range(h_kv)])
    x1 = store(x_g + linear(a.reshape(n_g, h_q * d), weights["w_o"]))
    h2 = store(rms_norm(x1, weights["ln2"], shape["rms_eps"]))
    x2 = store(x1 + swiglu_mlp(h2, weights["w_gate"], weights["w_up"], weights["w_down"], store))
    return x2, idx, new_k, new_v, dict(h=h, q=q, k=k, v=v, attn=a, scores=s, x1=x1, h2=h2)


def layer_stack(x, pos3, layers, shape, group_bounds, x_win, pos3_win, rule, retention, store=lambda t: t):
    """Group-major schedule of Sec. 3.2: every group runs through all layers before the next group starts;
    layer l keeps its own pruned cache. x [N, d_model]; layers: list of weight dicts; x_win [L, W, d_model]
    (or None for rules without a window). Returns the last layer's output and the per-layer caches."""
    x = np.asarray(x, dtype=np.float64)
    pos3 = np.asarray(pos3)
    h_kv, d = shape["n_kv_heads"], shape["head_dim"]
    caches = [(np.zeros((h_kv, 0, d)), np.zeros((h_kv, 0, d)), np.zeros((h_kv, 0), dtype=np.int64)) for _ in layers]
    q_wins = [None if x_win is None else window_queries(x_win[l], pos3_win, layers[l], shape, store)
              for l in range(len(layers))]
    out = np.zeros_like(x)
    for base, n_g in group_bounds:
        cur = x[base:base + n_g]
        for l, wts in enumerate(layers):
            ck, cv, cp = caches[l]
            cur, idx, nk, nv, _ = layer_group(cur, pos3[:, base:base + n_g], wts, shape, ck, cv, q_wins[l],
                                              rule, retention, store)
            caches[l] = (np.concatenate([ck, nk], axis=1), np.concatenate([cv, nv], axis=1),
                         np.concatenate([cp, base + idx], axis=1))
        out[base:base + n_g] = cur
    return out, caches
