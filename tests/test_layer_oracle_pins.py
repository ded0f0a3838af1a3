"""Pins for the decoder-layer oracle (oracle/layer_oracle.py): closed forms, invariants, library routines,
hand-computed cases. CPU only. Each test names the mistake it would catch."""
import math

import numpy as np
import pytest
import torch

from oracle import layer_oracle as lo
from oracle import qp_oracle as qo

RNG = np.random.default_rng(1234)


def small_shape(h_q=4, h_kv=2, d=8, d_model=12, sections=(1, 2, 1), theta=10000.0):
    return dict(n_q_heads=h_q, n_kv_heads=h_kv, head_dim=d, d_model=d_model, rms_eps=1e-6, rope_theta=theta,
                mrope_section=tuple(sections))


def random_layer(shape, d_ff=20, rng=RNG, zero_out=False):
    h_q, h_kv, d, dm = shape["n_q_heads"], shape["n_kv_heads"], shape["head_dim"], shape["d_model"]
    g = lambda *s: rng.standard_normal(s) / math.sqrt(s[-1])
    w = dict(ln1=1.0 + 0.1 * rng.standard_normal(dm), ln2=1.0 + 0.1 * rng.standard_normal(dm),
             w_q=g(h_q * d, dm), b_q=0.1 * rng.standard_normal(h_q * d),
             w_k=g(h_kv * d, dm), b_k=0.1 * rng.standard_normal(h_kv * d),
             w_v=g(h_kv * d, dm), b_v=0.1 * rng.standard_normal(h_kv * d),
             w_o=g(dm, h_q * d), w_gate=g(d_ff, dm), w_up=g(d_ff, dm), w_down=g(dm, d_ff))
    if zero_out:
        w["w_o"] = np.zeros_like(w["w_o"])
        w["w_down"] = np.zeros_like(w["w_down"])
    return w


# ----------------------------------------------------------------------------- bf16 rounding
def test_bf16_round_matches_library_and_ties_to_even():
    x = np.concatenate([RNG.standard_normal(4096) * 10.0 ** RNG.integers(-6, 6, 4096),
                        [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -1.0 - 2.0 ** -8, 0.0, 2.0 ** -130]])
    want = torch.tensor(x, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(lo.bf16_round(x), want)
    assert lo.bf16_round(1.0 + 2.0 ** -8) == 1.0                  # tie -> even mantissa (down)
    assert lo.bf16_round(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6   # tie -> even mantissa (up)


# ----------------------------------------------------------------------------- RMSNorm
def test_rms_norm_hand_case():
    # mean square of (3, 4) is 12.5
    y = lo.rms_norm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 0.0)
    np.testing.assert_allclose(y, [[3 / math.sqrt(12.5), 8 / math.sqrt(12.5)]], rtol=1e-15)


def test_rms_norm_invariants():
    x = RNG.standard_normal((5, 64))
    w = np.ones(64)
    y = lo.rms_norm(x, w, 0.0)
    np.testing.assert_allclose(np.mean(y * y, axis=-1), 1.0, rtol=1e-13)        # unit RMS (a mean/sum mix-up fails)
    np.testing.assert_allclose(lo.rms_norm(7.5 * x, w, 0.0), y, rtol=1e-13)     # scale invariance
    # no mean subtraction: a constant row stays constant and keeps its sign
    c = lo.rms_norm(np.full((1, 8), -2.0), np.ones(8), 0.0)
    np.testing.assert_allclose(c, -1.0, rtol=1e-15)
    # eps sits inside the square root, added to the mean (not to the root, not to the sum)
    e = lo.rms_norm(np.array([[1.0, 1.0, 1.0, 1.0]]), np.ones(4), 3.0)
    np.testing.assert_allclose(e, 0.5, rtol=1e-15)


def test_rms_norm_matches_library():
    x = torch.randn(7, 48, dtype=torch.float64)
    w = torch.randn(48, dtype=torch.float64)
    want = torch.nn.functional.rms_norm(x, (48,), w, 1e-6).numpy()
    np.testing.assert_allclose(lo.rms_norm(x.numpy(), w.numpy(), 1e-6), want, rtol=1e-13)


# ----------------------------------------------------------------------------- linear
def test_linear_hand_case_weight_is_out_by_in():
    w = np.array([[1.0, 2.0, 3.0], [0.0, -1.0, 1.0]])           # [out=2, in=3]
    y = lo.linear(np.array([[1.0, 1.0, 2.0]]), w, np.array([10.0, 20.0]))
    np.testing.assert_array_equal(y, [[19.0, 21.0]])


# ----------------------------------------------------------------------------- rotary embedding
def test_rotary_hand_case():
    # d = 4: frequency 0 = 1 (temporal axis), frequency 1 = theta^(-1/2) = 0.01 (height axis)
    cos, sin = lo.mrope_cos_sin(np.array([[math.pi / 2], [100.0], [7.0]]), 4, 10000.0, (1, 1, 0))
    y = lo.apply_rotary(np.array([[[1.0, 2.0, 3.0, 4.0]]]), cos, sin)
    want = [-3.0, 2 * math.cos(1.0) - 4 * math.sin(1.0), 1.0, 4 * math.cos(1.0) + 2 * math.sin(1.0)]
    np.testing.assert_allclose(y[0, 0], want, atol=1e-12)


def test_rotary_equal_axes_is_complex_rotation():
    d, n, theta = 16, 9, 1e6
    pos = RNG.integers(0, 5000, n)
    x = RNG.standard_normal((n, 3, d))
    cos, sin = lo.mrope_cos_sin(np.stack([pos, pos, pos]), d, theta, (3, 3, 2))
    y = lo.apply_rotary(x, cos, sin)
    z = (x[..., :d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * pos[:, None, None] *
                                                          theta ** (-np.arange(d // 2) / (d // 2)))[:, :, :]
    np.testing.assert_allclose(y[..., :d // 2], z.real, atol=1e-9)
    np.testing.assert_allclose(y[..., d // 2:], z.imag, atol=1e-9)


def test_rotary_relative_position_and_norm():
    d, sections = 16, (2, 3, 3)
    q = RNG.standard_normal((1, 1, d))
    k = RNG.standard_normal((1, 1, d))
    pq = np.array([[5], [11], [2]])
    pk = np.array([[3], [4], [9]])
    shift = np.array([[1000], [37], [512]])

    def dot(a, b):
        ca, sa = lo.mrope_cos_sin(a, d, 1e4, sections)
        cb, sb = lo.mrope_cos_sin(b, d, 1e4, sections)
        return float(np.sum(lo.apply_rotary(q, ca, sa) * lo.apply_rotary(k, cb, sb)))

    assert abs(dot(pq, pk) - dot(pq + shift, pk + shift)) < 1e-9       # only position differences matter
    assert abs(dot(pq, pk) - dot(pq, pk + 1)) > 1e-3                  # and they do matter
    c, s = lo.mrope_cos_sin(pq, d, 1e4, sections)
    np.testing.assert_allclose(np.linalg.norm(lo.apply_rotary(q, c, s)), np.linalg.norm(q), rtol=1e-13)
    # inverse rotation restores the vector (a sign slip in one of the two halves fails)
    cm, sm = lo.mrope_cos_sin(-pq, d, 1e4, sections)
    np.testing.assert_allclose(lo.apply_rotary(lo.apply_rotary(q, c, s), cm, sm), q, atol=1e-12)


def test_rotary_axis_sections():
    d, sections = 16, (2, 3, 3)
    x = RNG.standard_normal((1, 1, d))
    base = np.array([[4], [6], [8]])
    y0 = lo.apply_rotary(x, *lo.mrope_cos_sin(base, d, 1e4, sections))
    for axis, (lo_i, hi_i) in enumerate([(0, 2), (2, 5), (5, 8)]):
        p = base.copy()
        p[axis] += 3
        y = lo.apply_rotary(x, *lo.mrope_cos_sin(p, d, 1e4, sections))
        changed = np.abs(y - y0)[0, 0] > 1e-12
        want = np.zeros(d, dtype=bool)
        want[lo_i:hi_i] = True
        want[d // 2 + lo_i:d // 2 + hi_i] = True
        np.testing.assert_array_equal(changed, want)


# ----------------------------------------------------------------------------- SwiGLU (Appendix D.1)
def test_silu_closed_forms_and_library():
    assert lo.silu(0.0) == 0.0
    x = RNG.standard_normal(100) * 4
    np.testing.assert_allclose(lo.silu(x) - lo.silu(-x), x, atol=1e-13)          # x s(x) - (-x) s(-x) = x
    np.testing.assert_allclose(lo.silu(x), torch.nn.functional.silu(torch.tensor(x)).numpy(), rtol=1e-13)
    np.testing.assert_allclose(lo.silu(np.log(3.0)), np.log(3.0) * 0.75, rtol=1e-14)   # sigmoid(ln 3) = 3/4


def test_swiglu_hand_case_gate_takes_the_silu():
    # one input channel: gate 2, up 3, down 5 -> 5 * silu(2) * 3; swapping gate and up would give 5 * silu(3) * 2
    y = lo.swiglu_mlp(np.array([[1.0]]), np.array([[2.0]]), np.array([[3.0]]), np.array([[5.0]]))
    np.testing.assert_allclose(y, [[15.0 * 2.0 / (1.0 + math.exp(-2.0))]], rtol=1e-14)


# ----------------------------------------------------------------------------- the layer
def test_layer_is_identity_with_zero_output_projections():
    shape = small_shape()
    w = random_layer(shape, zero_out=True)
    x = RNG.standard_normal((6, shape["d_model"]))
    pos3 = np.stack([np.arange(6)] * 3)
    ck = np.zeros((2, 0, 8))
    y, idx, nk, nv, _ = lo.layer_group(x, pos3, w, shape, ck, ck, None, "key_norm_small", 0.5)
    np.testing.assert_array_equal(y, x)
    assert idx.shape == (2, 3) and nk.shape == (2, 3, 8)


def test_layer_single_token_attention_is_its_value():
    # one token, empty cache: softmax over one key is 1, so every query head returns the value of its KV head
    shape = small_shape()
    w = random_layer(shape)
    x = RNG.standard_normal((1, shape["d_model"]))
    pos3 = np.array([[17], [3], [5]])
    ck = np.zeros((2, 0, 8))
    _, _, _, _, mid = lo.layer_group(x, pos3, w, shape, ck, ck, None, "value_norm", 1.0)
    r = shape["n_q_heads"] // shape["n_kv_heads"]
    for qh in range(shape["n_q_heads"]):
        np.testing.assert_allclose(mid["attn"][0, qh], mid["v"][0, qh // r], rtol=1e-12)
    # v is not rotated, k is: |k| is preserved but k differs from the un-rotated projection
    k_raw = (mid["h"] @ w["w_k"].T + w["b_k"]).reshape(1, 2, 8)
    np.testing.assert_allclose(np.linalg.norm(mid["k"], axis=-1), np.linalg.norm(k_raw, axis=-1), rtol=1e-12)
    assert np.abs(mid["k"] - k_raw).max() > 1e-3
    np.testing.assert_allclose(mid["v"], (mid["h"] @ w["w_v"].T + w["b_v"]).reshape(1, 2, 8), rtol=1e-12)


def test_layer_attention_matches_library_sdpa():
    shape = small_shape()
    w = random_layer(shape)
    n = 10
    x = RNG.standard_normal((n, shape["d_model"]))
    pos3 = np.stack([np.arange(n), np.arange(n) % 3, np.arange(n) % 2])
    ck = np.zeros((2, 0, 8))
    _, _, _, _, mid = lo.layer_group(x, pos3, w, shape, ck, ck, None, "key_norm_small", 1.0)
    q = torch.tensor(mid["q"]).permute(1, 0, 2)[None]
    k = torch.tensor(mid["k"]).permute(1, 0, 2)[None].repeat_interleave(2, dim=1)
    v = torch.tensor(mid["v"]).permute(1, 0, 2)[None].repeat_interleave(2, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(mid["attn"], want, atol=1e-12)


@pytest.mark.parametrize("rule", ["key_norm_small", "window_attn"])
def test_stack_at_full_retention_equals_one_group(rule):
    """Sec. 3.2: group prefill with nothing pruned is ordinary causal prefill, so the group-major stack (keys
    rotated before they are cached, one cache per layer) must equal the whole sequence run as one group."""
    shape = small_shape()
    layers = [random_layer(shape), random_layer(shape), random_layer(shape)]
    tpf, frames = 4, 6
    n = tpf * frames
    x = RNG.standard_normal((n, shape["d_model"]))
    pos3 = np.stack([np.repeat(np.arange(frames), tpf), np.tile(np.arange(tpf) // 2, frames),
                     np.tile(np.arange(tpf) % 2, frames)])
    x_win = RNG.standard_normal((3, 5, shape["d_model"]))
    pos_win = np.stack([np.arange(5) + frames] * 3)
    grouped, caches = lo.layer_stack(x, pos3, layers, shape, qo.group_bounds(frames, tpf, 2), x_win, pos_win, rule, 1.0)
    whole, _ = lo.layer_stack(x, pos3, layers, shape, [(0, n)], x_win, pos_win, rule, 1.0)
    np.testing.assert_allclose(grouped, whole, atol=1e-10)
    for ck, cv, cp in caches:
        assert ck.shape == (2, n, 8)
        np.testing.assert_array_equal(cp, np.tile(np.arange(n), (2, 1)))


def test_stack_pruning_changes_later_groups_only():
    """With rho < 1 the first group's output is untouched (its cache is empty) and later groups differ."""
    shape = small_shape()
    layers = [random_layer(shape), random_layer(shape)]
    tpf, frames = 4, 4
    n = tpf * frames
    x = RNG.standard_normal((n, shape["d_model"]))
    pos3 = np.stack([np.arange(n)] * 3)
    gb = qo.group_bounds(frames, tpf, 2)
    full, _ = lo.layer_stack(x, pos3, layers, shape, gb, None, None, "key_norm_small", 1.0)
    pruned, caches = lo.layer_stack(x, pos3, layers, shape, gb, None, None, "key_norm_small", 0.5)
    np.testing.assert_allclose(pruned[:8], full[:8], atol=1e-12)
    assert np.abs(pruned[8:] - full[8:]).max() > 1e-6
    assert caches[0][0].shape == (2, 8, 8)


def test_store_hook_rounds_every_kept_tensor():
    shape = small_shape()
    w = random_layer(shape)
    x = lo.bf16_round(RNG.standard_normal((5, shape["d_model"])))
    pos3 = np.stack([np.arange(5)] * 3)
    ck = np.zeros((2, 0, 8))
    y, _, nk, nv, mid = lo.layer_group(x, pos3, w, shape, ck, ck, None, "key_norm_small", 0.6, store=lo.bf16_round)
    for name in ("h", "q", "k", "v", "attn", "x1", "h2"):
        np.testing.assert_array_equal(mid[name], lo.bf16_round(mid[name]), err_msg=name)
    np.testing.assert_array_equal(y, lo.bf16_round(y))
    np.testing.assert_array_equal(nk, lo.bf16_round(nk))
