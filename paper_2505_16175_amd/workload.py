"""Seeded synthetic video-token workloads for the QuickPrefill path.

This module only *generates inputs*; it contains none of the method's arithmetic
(no attention, scoring, selection or compaction) and is the one piece of code
that both the CPU oracle's tests and the HIP path's tests/benchmark may share.

The shapes mirror the paper's video workloads (a Qwen2.5-VL-7B-shaped layer:
28 query heads, 4 KV heads, head_dim 128; groups of 16-64 frames; retention
0.1-0.5, Sec. 4.2 / Table 1 / Table 2 / Sec. 4.3 of the paper); the values are
synthetic stand-ins for the activations of a trained model, which are not
available here.

Recipe for one layer, independently for Q, K and V (frame f, token slot t, head h):

    x[0, t, h, :] = eps                                    eps ~ N(0, 1) i.i.d.
    x[f, t, h, :] = a * x[f-1, t, h, :] + b * eps          inter-frame correlation (summed by doubling)
    K[n, :, :]   *= exp(sigma * z_n),  z_n ~ N(0, 1)       per-token log-normal key scale
    Q, K, V      /= sqrt(head_dim)
    Q_win[w, h, :] = N(0, 1) / sqrt(head_dim)              text-query window, uncorrelated
    (bf16 configs) round to nearest-even bf16

`sharp=True` drops the final 1/sqrt(head_dim) so that the attention logits have
O(1) spread; it exists for parity tests only (the literal recipe gives nearly
uniform softmax rows, which hide kernel mistakes).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import torch

BASE_SEED = 20250516


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" | "bf16"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_frames: int
    tokens_per_frame: int
    group_frames: int
    retention: float
    rules: tuple          # scoring rules this config runs, names as in the C-ABI enum
    n_window: int         # text-query window length W (0: none)
    corr_a: float         # AR(1) inter-frame coefficient
    corr_b: float         # fresh-noise coefficient
    key_sigma: float      # sigma of the LogNormal(0, sigma) per-token key scale
    n_layers: int = 1

    @property
    def n_tokens(self) -> int:
        return self.n_frames * self.tokens_per_frame

    @property
    def group_tokens(self) -> int:
        return self.group_frames * self.tokens_per_frame

    @property
    def gqa_ratio(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


# The five configurations the benchmark definition names, in its order.
CONFIGS = {
    "cfg1_tiny_f32": Workload("cfg1_tiny_f32", "f32", 4, 2, 64, 8, 16, 2, 0.5,
                              ("key_norm_small", "window_attn"), 16, 0.9, 0.44, 0.5),
    "cfg2_7b_32k": Workload("cfg2_7b_32k", "bf16", 28, 4, 128, 256, 128, 16, 0.3,
                            ("window_attn",), 64, 0.9, 0.44, 0.5),
    "cfg3_7b_128k_norm": Workload("cfg3_7b_128k_norm", "bf16", 28, 4, 128, 1024, 128, 32, 0.2,
                                  ("key_norm_small", "value_norm"), 0, 0.95,
                                  math.sqrt(1.0 - 0.95 ** 2), 0.5),
    "cfg4_72b_128k": Workload("cfg4_72b_128k", "bf16", 64, 8, 128, 512, 256, 16, 0.25,
                              ("window_attn",), 128, 0.9, 0.44, 0.75),
    "cfg5_7b_hour_stack": Workload("cfg5_7b_hour_stack", "bf16", 28, 4, 128, 3600, 128, 64, 0.1,
                                   ("window_attn",), 64, 0.9, 0.44, 0.5, n_layers=28),
}
CONFIG_ORDER = list(CONFIGS)


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a config with some fields replaced (smaller parity-test variants)."""
    return dataclasses.replace(w, **kw)


def _ar1(gen, n_frames, tokens_per_frame, n_heads, head_dim, a, b, device):
    """x[0] = eps[0], x[f] = a x[f-1] + b eps[f], i.e. x[f] = sum_j a^j u[f-j] with u[0] = eps[0], u[f] = b eps[f].
    Summed by doubling (after the pass with stride s every frame holds the terms j < 2s), so a video of F frames
    takes log2(F) passes over the tensor instead of F small ones."""
    x = torch.randn(n_frames, tokens_per_frame, n_heads, head_dim, generator=gen, dtype=torch.float32, device=device)
    x[1:] *= b
    stride = 1
    while stride < n_frames:
        nxt = x.clone()
        torch.add(x[stride:], x[:-stride], alpha=a ** stride, out=nxt[stride:])
        x = nxt
        stride *= 2
    return x.view(n_frames * tokens_per_frame, n_heads, head_dim)


def make_layer(w: Workload, layer: int = 0, device: str = "cpu", sharp: bool = False,
               seed: Optional[int] = None):
    """Q [N,H_q,d], K [N,H_kv,d], V [N,H_kv,d], Q_win [W,H_q,d] (or None) for one layer.

    Tensors are returned in the config's dtype on `device`. The random stream is
    that of a torch.Generator on `device` seeded with BASE_SEED + layer, so a CPU
    and a GPU generation of the same config differ in values (not in law); every
    comparison must therefore feed both sides from ONE call of this function.
    """
    gen = torch.Generator(device=device)
    gen.manual_seed((BASE_SEED if seed is None else seed) + layer)
    d = w.head_dim
    q = _ar1(gen, w.n_frames, w.tokens_per_frame, w.n_q_heads, d, w.corr_a, w.corr_b, device)
    k = _ar1(gen, w.n_frames, w.tokens_per_frame, w.n_kv_heads, d, w.corr_a, w.corr_b, device)
    v = _ar1(gen, w.n_frames, w.tokens_per_frame, w.n_kv_heads, d, w.corr_a, w.corr_b, device)
    z = torch.randn(w.n_tokens, generator=gen, dtype=torch.float32, device=device)
    k *= torch.exp(w.key_sigma * z).view(-1, 1, 1)
    qw = None
    if w.n_window > 0:
        qw = torch.randn(w.n_window, w.n_q_heads, d, generator=gen, dtype=torch.float32, device=device)
    if not sharp:
        s = 1.0 / math.sqrt(d)
        q *= s
        k *= s
        v *= s
        if qw is not None:
            qw *= s
    dt = w.torch_dtype()
    q, k, v = q.to(dt), k.to(dt), v.to(dt)
    if qw is not None:
        qw = qw.to(dt)
    return q, k, v, qw


def to_f64(t: Optional[torch.Tensor]):
    """Exact widening of an input tensor to a float64 numpy array on the host."""
    if t is None:
        return None
    return t.detach().to("cpu").to(torch.float64).numpy()


# ---- inputs of the decoder layer around the path (weights, hidden states, position indices) -----------------
@dataclasses.dataclass(frozen=True)
class LayerDims:
    """Sizes of a Qwen2.5-style decoder layer (head_dim 128)."""
    d_model: int
    d_ff: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    rms_eps: float = 1e-6
    rope_theta: float = 1e6
    mrope_section: tuple = (16, 24, 24)


LAYER_DIMS = {
    "7b": LayerDims(3584, 18944, 28, 4),
    "72b": LayerDims(8192, 29568, 64, 8),
}


def make_decoder_layer(dims: LayerDims, layer: int = 0, device: str = "cpu", seed: Optional[int] = None):
    """Random-init bf16 weights of one layer, [out][in]: N(0, 1/in) matrices, norm weights 1 + 0.1 N(0,1),
    biases 0.1 N(0,1). Keys: ln1_w, w_qkv (query heads, key heads, value heads), b_qkv, w_o, ln2_w,
    w_gate_up (gate rows, then up rows), w_down."""
    gen = torch.Generator(device=device)
    gen.manual_seed((BASE_SEED if seed is None else seed) + 7919 * (layer + 1))
    dm, dff = dims.d_model, dims.d_ff
    n_qkv = (dims.n_q_heads + 2 * dims.n_kv_heads) * dims.head_dim
    rn = lambda *s: torch.randn(*s, generator=gen, dtype=torch.float32, device=device)
    w = dict(ln1_w=1.0 + 0.1 * rn(dm), w_qkv=rn(n_qkv, dm) / math.sqrt(dm), b_qkv=0.1 * rn(n_qkv),
             w_o=rn(dm, dims.n_q_heads * dims.head_dim) / math.sqrt(dims.n_q_heads * dims.head_dim),
             ln2_w=1.0 + 0.1 * rn(dm), w_gate_up=rn(2 * dff, dm) / math.sqrt(dm), w_down=rn(dm, dff) / math.sqrt(dff))
    return {name: t.to(torch.bfloat16) for name, t in w.items()}


def make_hidden(n_frames, tokens_per_frame, d_model, corr_a=0.9, corr_b=0.44, device="cpu", seed=None):
    """Hidden states [N, d_model] entering a layer: N(0,1) channels with the same AR(1) inter-frame
    correlation as the Q/K/V recipe above, bf16."""
    gen = torch.Generator(device=device)
    gen.manual_seed((BASE_SEED if seed is None else seed) + 104729)
    return _ar1(gen, n_frames, tokens_per_frame, 1, d_model, corr_a, corr_b, device).view(-1, d_model).to(torch.bfloat16)


def video_positions(n_frames, tokens_per_frame, device="cpu", first_frame=0):
    """Position indices [3][N] int32 of a video's tokens: (frame index, row, column) of a token grid as square as
    tokens_per_frame allows (row-major inside a frame)."""
    gw = int(math.isqrt(tokens_per_frame))
    while tokens_per_frame % gw:
        gw -= 1
    slot = torch.arange(tokens_per_frame, dtype=torch.int32, device=device)
    t = torch.arange(first_frame, first_frame + n_frames, dtype=torch.int32, device=device).repeat_interleave(tokens_per_frame)
    return torch.stack([t, (slot // gw).repeat(n_frames), (slot % gw).repeat(n_frames)]).contiguous()


def text_positions(n_tokens, start, device="cpu"):
    """Text tokens carry the same index on all three axes."""
    p = torch.arange(start, start + n_tokens, dtype=torch.int32, device=device)
    return torch.stack([p, p, p]).contiguous()
