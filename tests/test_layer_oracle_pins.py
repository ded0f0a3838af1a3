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


# ----------------------------------------------------------------------------- the scoring window's queries
def test_window_queries_hand_case():
    """tests/golden/hand_window_queries.txt: one token through RMSNorm, W_q + b_q and the rotary embedding, every
    number worked by hand. Dropping the norm, the norm weight, the bias or the rotation, pairing neighbours instead of
    halves, or taking the wrong position axis for a frequency all change the numbers."""
    from conftest import read_golden
    rows = read_golden("hand_window_queries.txt")
    want_q = np.array([float(r[1]) for r in rows])
    want_rot = np.array([float(r[2]) for r in rows])
    shape = dict(n_q_heads=1, n_kv_heads=1, head_dim=4, d_model=4, rms_eps=0.0, rope_theta=100.0, mrope_section=(1, 1, 0))
    w = dict(ln1=np.array([1.0, 1.0, 2.0, 1.0]),
             w_q=np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0], [0, 0, 1.0, 0], [1.0, 1.0, 0, 0]]),
             b_q=np.array([0.0, 0.5, 0.0, -1.0]))
    x = np.array([[1.0, -1.0, 2.0, 0.0]])
    at_origin = lo.window_queries(x, np.array([[0], [0], [0]]), w, shape)      # angle 0: the projection itself
    np.testing.assert_allclose(at_origin[0, 0], want_q, atol=2e-15)
    got = lo.window_queries(x, np.array([[3], [5], [7]]), w, shape)
    assert got.shape == (1, 1, 4)
    np.testing.assert_allclose(got[0, 0], want_rot, atol=3e-15)
    # project_queries is the part after the norm
    h = np.array([[1.0, -1.0, 4.0, 0.0]]) / math.sqrt(1.5)
    np.testing.assert_allclose(lo.project_queries(h, w["w_q"], w["b_q"], np.array([[3], [5], [7]]), shape)[0, 0],
                               want_rot, atol=3e-15)


def test_window_queries_invariants():
    shape = small_shape()
    w = random_layer(shape)
    n = 5
    x = RNG.standard_normal((n, shape["d_model"]))
    pos = np.stack([np.arange(n) + 9, np.arange(n) + 2, np.arange(n)])
    q = lo.window_queries(x, pos, w, shape)
    assert q.shape == (n, shape["n_q_heads"], shape["head_dim"])
    # the hidden states are normalised first: scaling them changes nothing (fails if RMSNorm is dropped)
    no_eps = dict(shape, rms_eps=0.0)
    np.testing.assert_allclose(lo.window_queries(3.7 * x, pos, w, no_eps), lo.window_queries(x, pos, w, no_eps),
                               rtol=1e-12, atol=1e-13)
    # it is the FIRST norm's weight, and only the query projection's parameters
    w2 = dict(w, ln2=w["ln2"] * 3.0, w_k=w["w_k"] * 2.0, b_k=w["b_k"] + 1.0, w_v=w["w_v"] * 2.0, w_o=w["w_o"] * 2.0)
    np.testing.assert_array_equal(lo.window_queries(x, pos, w2, shape), q)
    assert np.abs(lo.window_queries(x, pos, dict(w, ln1=w["ln1"] * 1.5), shape) - q).max() > 1e-3
    # the bias is added before the rotation: with a zero matrix the queries are the rotated bias, at the origin the bias itself
    wz = dict(w, w_q=np.zeros_like(w["w_q"]))
    at0 = lo.window_queries(x, np.zeros((3, n), dtype=np.int64), wz, shape)
    np.testing.assert_allclose(at0, np.broadcast_to(w["b_q"].reshape(1, shape["n_q_heads"], -1), at0.shape), atol=1e-15)
    rot = lo.window_queries(x, pos, wz, shape)
    np.testing.assert_allclose(np.linalg.norm(rot, axis=-1), np.linalg.norm(at0, axis=-1), rtol=1e-12)
    assert np.abs(rot - at0).max() > 1e-3
    # rotation is per token: the queries of token i do not depend on the other tokens
    np.testing.assert_allclose(lo.window_queries(x[2:3], pos[:, 2:3], w, shape), q[2:3], atol=1e-14)


def test_window_queries_equal_the_layers_own_queries_for_the_same_tokens():
    # the window's tokens run as a group through the same layer produce the same q (same norm, projection, rotation)
    shape = small_shape()
    w = random_layer(shape)
    n = 6
    x = RNG.standard_normal((n, shape["d_model"]))
    pos = np.stack([np.arange(n) + 40, np.arange(n) + 40, np.arange(n) + 40])
    empty = np.zeros((shape["n_kv_heads"], 0, shape["head_dim"]))
    _, _, _, _, mid = lo.layer_group(x, pos, w, shape, empty, empty, None, "key_norm_small", 1.0)
    np.testing.assert_allclose(lo.window_queries(x, pos, w, shape), mid["q"], atol=1e-14)
    # and with the storage hook both round at the same places
    _, _, _, _, mid_r = lo.layer_group(lo.bf16_round(x), pos, w, shape, empty, empty, None, "key_norm_small", 1.0,
                                       store=lo.bf16_round)
    np.testing.assert_array_equal(lo.window_queries(lo.bf16_round(x), pos, w, shape, store=lo.bf16_round), mid_r["q"])


# ----------------------------------------------------------------------------- the block's wiring
def _torch_block(x, pos1d, w, shape):
    """The same pre-norm block out of library routines only (torch.nn.functional rms_norm / linear / silu /
    scaled_dot_product_attention, rotation as a complex multiplication), one group, empty cache, equal position
    indices on the three axes."""
    F = torch.nn.functional
    t = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    n, dm = x.shape
    h_q, h_kv, d = shape["n_q_heads"], shape["n_kv_heads"], shape["head_dim"]
    half = d // 2
    rot = torch.polar(torch.ones(n, half, dtype=torch.float64),
                      t(pos1d)[:, None] * shape["rope_theta"] ** (-2.0 * torch.arange(half, dtype=torch.float64) / d))

    def rotate(z):                                              # [n, H, d]; component i pairs with i + d/2
        zc = torch.complex(z[..., :half], z[..., half:]) * rot[:, None, :]
        return torch.cat([zc.real, zc.imag], dim=-1)

    xt = t(x)
    h = F.rms_norm(xt, (dm,), t(w["ln1"]), shape["rms_eps"])
    q = rotate(F.linear(h, t(w["w_q"]), t(w["b_q"])).view(n, h_q, d))
    k = rotate(F.linear(h, t(w["w_k"]), t(w["b_k"])).view(n, h_kv, d))
    v = F.linear(h, t(w["w_v"]), t(w["b_v"])).view(n, h_kv, d)
    r = h_q // h_kv
    a = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None].repeat_interleave(r, dim=1),
                                       v.permute(1, 0, 2)[None].repeat_interleave(r, dim=1), is_causal=True)
    a = a[0].permute(1, 0, 2).reshape(n, h_q * d)
    x1 = xt + F.linear(a, t(w["w_o"]))
    h2 = F.rms_norm(x1, (dm,), t(w["ln2"]), shape["rms_eps"])
    x2 = x1 + F.linear(F.silu(F.linear(h2, t(w["w_gate"]))) * F.linear(h2, t(w["w_up"])), t(w["w_down"]))
    return x1.numpy(), h2.numpy(), x2.numpy()


def test_layer_block_equals_the_same_block_built_from_library_routines():
    """Catches any mis-wiring of the residual stream: the second norm or the MLP fed from x instead of x1, a
    residual dropped or doubled, the two norm weights swapped, gate and up exchanged."""
    shape = small_shape()
    w = random_layer(shape)
    n = 9
    x = RNG.standard_normal((n, shape["d_model"]))
    p = np.arange(n) + 3
    empty = np.zeros((shape["n_kv_heads"], 0, shape["head_dim"]))
    y, _, _, _, mid = lo.layer_group(x, np.stack([p, p, p]), w, shape, empty, empty, None, "key_norm_small", 1.0)
    x1, h2, x2 = _torch_block(x, p, w, shape)
    np.testing.assert_allclose(mid["x1"], x1, atol=1e-12)
    np.testing.assert_allclose(mid["h2"], h2, atol=1e-12)
    np.testing.assert_allclose(y, x2, atol=1e-12)


def test_layer_block_composed_from_its_parts_and_perturbations():
    shape = small_shape()
    w = random_layer(shape)
    n = 7
    x = RNG.standard_normal((n, shape["d_model"]))
    pos = np.stack([np.arange(n), np.arange(n) % 2, np.arange(n) % 3])
    ck = RNG.standard_normal((shape["n_kv_heads"], 5, shape["head_dim"]))      # a non-empty cache this time
    cv = RNG.standard_normal((shape["n_kv_heads"], 5, shape["head_dim"]))
    run = lambda wt: lo.layer_group(x, pos, wt, shape, ck, cv, None, "value_norm", 0.5)
    y, _, _, _, mid = run(w)
    # composition by hand from the pinned parts
    x1 = x + lo.linear(mid["attn"].reshape(n, -1), w["w_o"])
    h2 = lo.rms_norm(x1, w["ln2"], shape["rms_eps"])
    x2 = x1 + lo.swiglu_mlp(h2, w["w_gate"], w["w_up"], w["w_down"])
    np.testing.assert_allclose(mid["x1"], x1, atol=1e-14)
    np.testing.assert_allclose(mid["h2"], h2, atol=1e-14)
    np.testing.assert_allclose(y, x2, atol=1e-14)
    # the second norm and the MLP see the attention's contribution; the first residual does not see the second norm
    _, _, _, _, m_o = run(dict(w, w_o=w["w_o"] * 1.5))
    assert np.abs(m_o["h2"] - mid["h2"]).max() > 1e-3 and np.abs(m_o["x1"] - mid["x1"]).max() > 1e-3
    y_ln2, _, _, _, m_ln2 = run(dict(w, ln2=w["ln2"] * 1.5))
    np.testing.assert_array_equal(m_ln2["x1"], mid["x1"])
    assert np.abs(y_ln2 - y).max() > 1e-3
    # the MLP's output is added to x1 (not to x): with w_down = 0 the layer returns x1
    y0, _, _, _, m0 = run(dict(w, w_down=np.zeros_like(w["w_down"])))
    np.testing.assert_array_equal(y0, m0["x1"])
    assert np.abs(m0["x1"] - x).max() > 1e-3
    # and with w_o = 0 it is x + MLP(RMSNorm(x; ln2))
    yo, _, _, _, _ = run(dict(w, w_o=np.zeros_like(w["w_o"])))
    np.testing.assert_allclose(yo, x + lo.swiglu_mlp(lo.rms_norm(x, w["ln2"], shape["rms_eps"]), w["w_gate"], w["w_up"],
                                                     w["w_down"]), atol=1e-14)
    # the cache is read by the attention: other cached values change the output, the kept rows come from this group's k, v
    y_c, idx, nk, nv, m_c = lo.layer_group(x, pos, w, shape, ck, cv * 2.0, None, "value_norm", 0.5)
    assert np.abs(y_c - y).max() > 1e-3
    for j in range(shape["n_kv_heads"]):
        np.testing.assert_array_equal(nk[j], m_c["k"][idx[j], j])
        np.testing.assert_array_equal(nv[j], m_c["v"][idx[j], j])


@pytest.mark.parametrize("rule", ["window_attn", "window_logit"])
def test_stack_window_rule_selects_on_this_layers_own_window_queries(rule):
    """With rho < 1 the window rule decides what is kept: the kept indices of every layer must be the top-k of
    score_kv over that layer's own keys and that layer's own window queries (not another layer's, not unrotated)."""
    shape = small_shape()
    layers = [random_layer(shape), random_layer(shape)]
    tpf, frames = 4, 4
    n = tpf * frames
    x = RNG.standard_normal((n, shape["d_model"]))
    pos3 = np.stack([np.repeat(np.arange(frames), tpf), np.tile(np.arange(tpf), frames), np.zeros(n, dtype=np.int64)])
    x_win = RNG.standard_normal((2, 3, shape["d_model"]))
    pos_win = np.stack([np.arange(3) + frames] * 3)
    gb = qo.group_bounds(frames, tpf, 2)
    _, caches = lo.layer_stack(x, pos3, layers, shape, gb, x_win, pos_win, rule, 0.5)
    # replay by hand, group-major: every group goes through layer 0 then layer 1; layer l scores its own keys with its
    # own window queries (its own text hidden states through its own norm and W_q)
    empty = np.zeros((2, 0, 8))
    state = [[empty, empty, []] for _ in layers]
    for base, n_g in gb:
        cur = x[base:base + n_g]
        for l, wts in enumerate(layers):
            qw = lo.window_queries(x_win[l], pos_win, wts, shape)
            ck, cv, kept_l = state[l]
            cur, idx, nk, nv, mid = lo.layer_group(cur, pos3[:, base:base + n_g], wts, shape, ck, cv, qw, rule, 0.5)
            want = qo.topk_select(qo.score_kv(rule, mid["k"], mid["v"], qw), qo.keep_count(n_g, 0.5))
            np.testing.assert_array_equal(idx, want)
            kept_l.append(base + idx)
            state[l][0], state[l][1] = np.concatenate([ck, nk], axis=1), np.concatenate([cv, nv], axis=1)
    for l in range(len(layers)):
        np.testing.assert_array_equal(caches[l][2], np.concatenate(state[l][2], axis=1))
        np.testing.assert_array_equal(caches[l][0], state[l][0])
    kept = state[0][2]
    # another layer's window queries would have kept something else somewhere
    qw_other = lo.window_queries(x_win[1], pos_win, layers[0], shape)
    _, idx_other, _, _, _ = lo.layer_group(x[:8], pos3[:, :8], layers[0], shape, empty, empty, qw_other, rule, 0.5)
    assert not np.array_equal(idx_other, kept[0])
