"""GPU parity of the decoder layer around the path (include/qp_layer.h) against the fp64 layer oracle."""
import numpy as np
import pytest
import torch

from oracle import layer_oracle as LO
from oracle import qp_oracle as O
from paper_2505_16175_amd import binding as B
from paper_2505_16175_amd import workload as W
from paper_2505_16175_amd.workload import to_f64
from helpers import assert_layer_close, compare_kept, oracle_shape, oracle_weights

pytestmark = pytest.mark.gpu
DEV = "cuda"

# A stored bf16 value is the rounding of an f32-accumulated sum; the oracle rounds the exact sum at the same place.
# The two differ only where the f32 and the exact value straddle a rounding boundary: one bf16 ulp (<= 2^-7 of the
# value). The absolute floor covers outputs that are small by cancellation (f32 summation error relative to the
# tensor's RMS). A wrong index, operand or epilogue produces errors of the size of the RMS itself.
def assert_stored_close(got, want, what, ulps=1.0, floor=2e-4, nrm=3e-3):
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    rms = np.sqrt(np.mean(want * want))
    err = np.abs(got - want)
    bad = err > ulps * 2.0 ** -7 * np.abs(want) + floor * rms
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} out of tolerance, max err {err.max():.3e} (rms {rms:.3e})"
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    assert rel <= nrm, f"{what}: normalised error {rel:.3e}"
    return rel


@pytest.fixture(params=[128, 256, 0], ids=["tile128", "tile256", "tile_auto"])
def tile(request):
    """Every projection test runs with both workgroup tilings forced, and with the launcher's own choice."""
    B.select_linear_tile(request.param)
    yield request.param
    B.select_linear_tile(0)


def _bf(*shape, gen, scale=1.0):
    return (torch.randn(*shape, generator=gen) * scale).to(torch.bfloat16)


@pytest.mark.parametrize("n,d", [(1, 64), (5, 3584), (300, 256), (257, 8192), (4, 72), (3, 8200), (2, 16384)])
def test_rms_norm(n, d):
    print(f"case n={n} d={d}", flush=True)
    g = torch.Generator().manual_seed(n * 131 + d)
    x, w = _bf(n, d, gen=g, scale=3.0), (1.0 + 0.1 * torch.randn(d, generator=g)).to(torch.bfloat16)
    out = torch.full((n, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.rms_norm(x.to(DEV), w.to(DEV), out, 1e-6)
    torch.cuda.synchronize()
    assert_stored_close(to_f64(out), LO.bf16_round(LO.rms_norm(to_f64(x), to_f64(w), 1e-6)), "rms_norm")


@pytest.mark.parametrize("m,n,k,bias,res", [(1, 8, 64, False, False), (300, 512, 192, True, True), (257, 200, 128, True, False),
                                            (256, 256, 64, False, True), (513, 264, 3584, True, True),
                                            (40, 3584, 18944, False, True), (1000, 1024, 320, False, False),
                                            (40, 8192, 29568, False, True)])
def test_linear(m, n, k, bias, res, tile):
    print(f"case m={m} n={n} k={k} bias={bias} residual={res}", flush=True)
    g = torch.Generator().manual_seed(m + 7 * n + 13 * k)
    x, w = _bf(m, k, gen=g), _bf(n, k, gen=g, scale=k ** -0.5)
    b = _bf(n, gen=g, scale=0.5) if bias else None
    r = _bf(m, n, gen=g) if res else None
    want = LO.linear(to_f64(x), to_f64(w), None if b is None else to_f64(b))
    if r is not None:
        want = want + to_f64(r)
    out = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
    dv = lambda t: None if t is None else t.to(DEV)
    B.linear(dv(x), dv(w), dv(b), dv(r), out)
    torch.cuda.synchronize()
    assert_stored_close(to_f64(out), LO.bf16_round(want), "linear")
    if r is not None:   # the residual may alias the output
        out2 = r.to(DEV).clone()
        B.linear(dv(x), dv(w), dv(b), out2, out2)
        torch.cuda.synchronize()
        assert torch.equal(out2, out)


@pytest.mark.parametrize("n,theta,sections", [(300, 1e6, (16, 24, 24)), (7, 1e4, (64, 0, 0)), (1025, 1e6, (0, 32, 32))])
def test_rope_table(n, theta, sections):
    print(f"case n={n} theta={theta} sections={sections}", flush=True)
    g = torch.Generator().manual_seed(n)
    pos = torch.stack([torch.randint(0, 100000, (n + 9,), generator=g), torch.randint(0, 64, (n + 9,), generator=g),
                       torch.randint(0, 64, (n + 9,), generator=g)]).to(torch.int32)
    cs = torch.full((n, 64, 2), float("nan"), dtype=torch.float32, device=DEV)
    B.rope_table(pos.to(DEV), 4, n, theta, sections, cs)          # a slice of a longer [3][N] array
    torch.cuda.synchronize()
    cos, sin = LO.mrope_cos_sin(pos[:, 4:4 + n].numpy(), 128, theta, sections)
    got = to_f64(cs)
    # the angle is formed in f64 on both sides; f32 rounding of the result is all that is left (+ theta as f32)
    np.testing.assert_allclose(got[..., 0], cos, atol=2e-7 if theta == 1e6 or theta == 1e4 else 1e-4, rtol=0)
    np.testing.assert_allclose(got[..., 1], sin, atol=2e-7 if theta == 1e6 or theta == 1e4 else 1e-4, rtol=0)


def _oracle_qkv(h, w_qkv, b_qkv, pos3, h_q, h_kv, theta, sections):
    n = h.shape[0]
    y = LO.linear(h, w_qkv, b_qkv)
    cos, sin = LO.mrope_cos_sin(pos3, 128, theta, sections)
    q = LO.apply_rotary(y[:, :h_q * 128].reshape(n, h_q, 128), cos, sin)
    k = LO.apply_rotary(y[:, h_q * 128:(h_q + h_kv) * 128].reshape(n, h_kv, 128), cos, sin)
    v = y[:, (h_q + h_kv) * 128:].reshape(n, h_kv, 128)
    return LO.bf16_round(q), LO.bf16_round(k), LO.bf16_round(v)


@pytest.mark.parametrize("n,d_model,h_q,h_kv", [(300, 320, 4, 2), (1, 64, 2, 1), (257, 3584, 28, 4), (600, 192, 6, 3),
                                                (130, 512, 8, 8), (130, 8192, 64, 8)])
def test_qkv_rope(n, d_model, h_q, h_kv, tile):
    print(f"case n={n} d_model={d_model} heads={h_q}/{h_kv}", flush=True)
    g = torch.Generator().manual_seed(n + d_model + h_q)
    theta, sections = 1e6, (16, 24, 24)
    h = _bf(n, d_model, gen=g)
    nq = (h_q + 2 * h_kv) * 128
    w, b = _bf(nq, d_model, gen=g, scale=d_model ** -0.5), _bf(nq, gen=g, scale=0.5)
    pos = W.video_positions((n + 15) // 16, 16)[:, :n].contiguous()
    pos[0] += 3000                                              # long-video temporal indices
    want = _oracle_qkv(to_f64(h), to_f64(w), to_f64(b), pos.numpy(), h_q, h_kv, theta, sections)
    layout = B.make_layout(h_q, h_kv, 128, "bf16")
    cs = torch.empty(n, 64, 2, dtype=torch.float32, device=DEV)
    B.rope_table(pos.to(DEV), 0, n, theta, sections, cs)
    q = torch.full((n, h_q, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    k = torch.full((n, h_kv, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    v = torch.full((n, h_kv, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.qkv_rope(layout, h.to(DEV), w.to(DEV), b.to(DEV), cs, q, k, v)
    torch.cuda.synchronize()
    for name, got, ref in zip("qkv", (q, k, v), want):
        assert_stored_close(to_f64(got), ref, name)


@pytest.mark.parametrize("n,d_model,d_ff", [(300, 192, 384), (1, 64, 128), (257, 3584, 18944), (513, 256, 1152),
                                            (48, 8192, 29568)])
def test_swiglu_gate_up(n, d_model, d_ff, tile):
    print(f"case n={n} d_model={d_model} d_ff={d_ff}", flush=True)
    g = torch.Generator().manual_seed(n + d_model + d_ff)
    h = _bf(n, d_model, gen=g)
    w = _bf(2 * d_ff, d_model, gen=g, scale=2.0 * d_model ** -0.5)
    want = LO.silu(LO.linear(to_f64(h), to_f64(w[:d_ff]))) * LO.linear(to_f64(h), to_f64(w[d_ff:]))
    act = torch.full((n, d_ff), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.swiglu_gate_up(h.to(DEV), w.to(DEV), act)
    torch.cuda.synchronize()
    # exp and the division add a few f32 ulps before the rounding: still far inside one bf16 ulp
    assert_stored_close(to_f64(act), LO.bf16_round(want), "swiglu")


@pytest.mark.parametrize("m", [1, 2])
@pytest.mark.parametrize("d_model,d_ff,h_q,h_kv", [(3584, 18944, 28, 4), (192, 384, 6, 3), (8192, 29568, 64, 8)])
def test_few_token_projections_stream_the_weights(m, d_model, d_ff, h_q, h_kv):
    """Calls of at most 2 tokens (decoding through the layer, Sec. 2.1) take the kernel that streams the weights once:
    all three stores against the oracle at the layer's real sizes, agreement with the tiled kernel at bf16 level, and
    the plan says which kernel runs."""
    print(f"case m={m} d_model={d_model} d_ff={d_ff} heads={h_q}/{h_kv}", flush=True)
    g = torch.Generator().manual_seed(m + d_model + d_ff)
    dv = lambda t: t.to(DEV)
    plan = B.linear_plan(m, d_model, d_ff, 32 << 20)
    assert plan["token_rows_per_tile"] == m and plan["k_chunks"] == 1
    assert plan["workgroups"] == d_model // 4 and plan["scratch_bytes"] == 0
    # down projection with residual, o_proj-shaped projection with bias
    for n, k, bias in ((d_model, d_ff, False), (d_model, h_q * 128, True)):
        x, w = _bf(m, k, gen=g), _bf(n, k, gen=g, scale=k ** -0.5)
        b = _bf(n, gen=g, scale=0.5) if bias else None
        r = _bf(m, n, gen=g)
        want = LO.linear(to_f64(x), to_f64(w), None if b is None else to_f64(b)) + to_f64(r)
        out = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
        B.linear(dv(x), dv(w), None if b is None else dv(b), dv(r), out)
        torch.cuda.synchronize()
        assert_stored_close(to_f64(out), LO.bf16_round(want), f"streamed linear k={k}")
        B.select_linear_tile(256)
        try:
            assert B.linear_plan(m, n, k, 0)["token_rows_per_tile"] == 256
            tiled = torch.full_like(out, float("nan"))
            B.linear(dv(x), dv(w), None if b is None else dv(b), dv(r), tiled)
            torch.cuda.synchronize()
        finally:
            B.select_linear_tile(0)
        assert_stored_close(to_f64(tiled), LO.bf16_round(want), f"tiled linear k={k}")
        out2 = dv(r).clone()                                      # the residual may alias the output
        B.linear(dv(x), dv(w), None if b is None else dv(b), out2, out2)
        torch.cuda.synchronize()
        assert torch.equal(out2, out)
    # QKV + bias + rotary embedding
    theta, sections = 1e6, (16, 24, 24)
    h = _bf(m, d_model, gen=g)
    nq = (h_q + 2 * h_kv) * 128
    w, b = _bf(nq, d_model, gen=g, scale=d_model ** -0.5), _bf(nq, gen=g, scale=0.5)
    pos = W.text_positions(m, 46000)
    want = _oracle_qkv(to_f64(h), to_f64(w), to_f64(b), pos.numpy(), h_q, h_kv, theta, sections)
    layout = B.make_layout(h_q, h_kv, 128, "bf16")
    cs = torch.empty(m, 64, 2, dtype=torch.float32, device=DEV)
    B.rope_table(pos.to(DEV), 0, m, theta, sections, cs)
    q = torch.full((m, h_q, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    k = torch.full((m, h_kv, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    v = torch.full((m, h_kv, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.qkv_rope(layout, dv(h), dv(w), dv(b), cs, q, k, v)
    torch.cuda.synchronize()
    for name, got, ref in zip("qkv", (q, k, v), want):
        assert_stored_close(to_f64(got), ref, f"streamed {name}")
    # SwiGLU gate / up
    w = _bf(2 * d_ff, d_model, gen=g, scale=2.0 * d_model ** -0.5)
    want = LO.silu(LO.linear(to_f64(h), to_f64(w[:d_ff]))) * LO.linear(to_f64(h), to_f64(w[d_ff:]))
    act = torch.full((m, d_ff), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.swiglu_gate_up(dv(h), dv(w), act)
    torch.cuda.synchronize()
    assert_stored_close(to_f64(act), LO.bf16_round(want), "streamed swiglu")


@pytest.mark.parametrize("m,n,k,bias,res", [(1, 3584, 18944, False, True), (7, 512, 1024, True, True), (64, 3584, 3584, False, True),
                                            (130, 264, 640, True, False), (300, 1024, 4096, False, False)])
def test_linear_split_contraction(m, n, k, bias, res):
    """Few tokens against long rows with scratch offered: the contraction is dealt to k chunks and a second launch
    adds the partial sums. Same tolerance as the unsplit call, and bit-identical between two runs."""
    print(f"case m={m} n={n} k={k}", flush=True)
    g = torch.Generator().manual_seed(m + 3 * n + 5 * k)
    x, w = _bf(m, k, gen=g), _bf(n, k, gen=g, scale=k ** -0.5)
    b = _bf(n, gen=g, scale=0.5) if bias else None
    r = _bf(m, n, gen=g) if res else None
    want = LO.linear(to_f64(x), to_f64(w), None if b is None else to_f64(b))
    if r is not None:
        want = want + to_f64(r)
    dv = lambda t: None if t is None else t.to(DEV)
    scratch = torch.empty(32 << 20, dtype=torch.uint8, device=DEV)
    outs = []
    if m <= 2:
        B.select_linear_tile(256)      # a handful of tokens would otherwise take the weight-streaming kernel
    try:
        assert B.linear_plan(m, n, k, 32 << 20)["k_chunks"] > 1
        for _ in range(2):
            out = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
            scratch.fill_(0xff)                                   # NaN patterns: every partial read must have been written
            B.linear(dv(x), dv(w), dv(b), dv(r), out, scratch)
            torch.cuda.synchronize()
            outs.append(out)
    finally:
        B.select_linear_tile(0)
    assert_stored_close(to_f64(outs[0]), LO.bf16_round(want), "split linear")
    assert torch.equal(outs[0], outs[1])
    plain = torch.empty_like(outs[0])
    B.linear(dv(x), dv(w), dv(b), dv(r), plain)                   # unsplit: differs at most by rounding flips
    torch.cuda.synchronize()
    assert_stored_close(to_f64(plain), LO.bf16_round(want), "unsplit linear")


@pytest.mark.parametrize("n,d_model,h_q,h_kv", [(1, 3584, 28, 4), (9, 1024, 4, 2), (64, 3584, 28, 4)])
def test_qkv_rope_split_contraction(n, d_model, h_q, h_kv):
    print(f"case n={n} d_model={d_model} heads={h_q}/{h_kv}", flush=True)
    g = torch.Generator().manual_seed(7 * n + d_model + h_q)
    theta, sections = 1e6, (16, 24, 24)
    h = _bf(n, d_model, gen=g)
    nq = (h_q + 2 * h_kv) * 128
    w, b = _bf(nq, d_model, gen=g, scale=d_model ** -0.5), _bf(nq, gen=g, scale=0.5)
    pos = W.text_positions(n, 4000)
    want = _oracle_qkv(to_f64(h), to_f64(w), to_f64(b), pos.numpy(), h_q, h_kv, theta, sections)
    layout = B.make_layout(h_q, h_kv, 128, "bf16")
    cs = torch.empty(n, 64, 2, dtype=torch.float32, device=DEV)
    B.rope_table(pos.to(DEV), 0, n, theta, sections, cs)
    scratch = torch.empty(32 << 20, dtype=torch.uint8, device=DEV)
    scratch.fill_(0xff)
    q = torch.full((n, h_q, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    k = torch.full((n, h_kv, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    v = torch.full((n, h_kv, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    if n <= 2:
        B.select_linear_tile(256)      # a handful of tokens would otherwise take the weight-streaming kernel
    try:
        B.qkv_rope(layout, h.to(DEV), w.to(DEV), b.to(DEV), cs, q, k, v, scratch)
        torch.cuda.synchronize()
    finally:
        B.select_linear_tile(0)
    for name, got, ref in zip("qkv", (q, k, v), want):
        assert_stored_close(to_f64(got), ref, name)


def test_unsupported_shapes_are_refused_before_launch():
    x = torch.zeros(4, 72, dtype=torch.bfloat16, device=DEV)
    w = torch.zeros(8, 72, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(4, 8, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.QPError) as e:
        B.linear(x, w, None, None, out)                          # k not a multiple of 64
    assert e.value.status == B.QP_ERR_UNSUPPORTED
    with pytest.raises(B.QPError) as e:
        B.swiglu_gate_up(torch.zeros(4, 64, dtype=torch.bfloat16, device=DEV),
                         torch.zeros(2 * 64, 64, dtype=torch.bfloat16, device=DEV),
                         torch.zeros(4, 64, dtype=torch.bfloat16, device=DEV))   # d_ff not a multiple of 128
    assert e.value.status == B.QP_ERR_UNSUPPORTED


# ------------------------------------------------------------------------------------------------ the layer
def _gpu_stack(dims, layers_t, x, pos, bounds, x_win, pos_win, rule, retention):
    """The group-major schedule of Sec. 3.2 driven through the C ABI: every group runs through all layers."""
    layout = B.make_layout(dims.n_q_heads, dims.n_kv_heads, 128, "bf16")
    shape = B.make_layer_shape(dims.d_model, dims.d_ff, dims.rms_eps, dims.rope_theta, dims.mrope_section)
    n_win = 0 if x_win is None else x_win.shape[1]
    n_max = max(n for _, n in bounds)
    ws = B.make_layer_workspace(layout, shape, n_max, n_win)
    weights = [B.LayerWeights(**{k: v.to(DEV) for k, v in w.items()}) for w in layers_t]
    cap = sum(B.keep_count(n, retention) for _, n in bounds)
    caches = [B.Cache(layout, cap) for _ in layers_t]
    q_wins = [None] * len(layers_t)
    if x_win is not None:
        pw = pos_win.to(DEV)
        for l, wt in enumerate(weights):
            q_wins[l] = torch.empty(n_win, dims.n_q_heads, 128, dtype=torch.bfloat16, device=DEV)
            B.layer_window_queries(layout, shape, wt, x_win[l].to(DEV), pw, q_wins[l], ws)
    xd, pd = x.to(DEV), pos.to(DEV)
    out = torch.empty_like(xd)
    kept = []
    for base, n_g in bounds:
        cur = xd[base:base + n_g].contiguous()
        keep = B.keep_count(n_g, retention)
        for l, wt in enumerate(weights):
            idx = torch.empty(dims.n_kv_heads, keep, dtype=torch.int32, device=DEV)
            nxt = torch.empty_like(cur)
            B.layer_group(layout, shape, wt, cur, pd, base, base, q_wins[l], rule, keep, caches[l], nxt, idx, ws)
            kept.append((base, l, idx))
            cur = nxt
        out[base:base + n_g] = cur
    torch.cuda.synchronize()
    return out, caches, kept


def _gpu_group_qkv(dims, wt_dev, x_dev, pos_dev, first, n_g):
    """The group's rotated q, k and its v as the layer computes them on the GPU (same calls, same kernels: RMSNorm,
    rotary table, fused QKV projection with the contraction-split scratch the layer offers), returned widened."""
    layout = B.make_layout(dims.n_q_heads, dims.n_kv_heads, 128, "bf16")
    h = torch.empty_like(x_dev)
    cs = torch.empty(n_g, 64, 2, dtype=torch.float32, device=DEV)
    q = torch.empty(n_g, dims.n_q_heads, 128, dtype=torch.bfloat16, device=DEV)
    k = torch.empty(n_g, dims.n_kv_heads, 128, dtype=torch.bfloat16, device=DEV)
    v = torch.empty_like(k)
    scratch = torch.empty(32 << 20, dtype=torch.uint8, device=DEV)
    B.rms_norm(x_dev, wt_dev["ln1_w"], h, dims.rms_eps)
    B.rope_table(pos_dev, first, n_g, dims.rope_theta, dims.mrope_section, cs)
    B.qkv_rope(layout, h, wt_dev["w_qkv"], wt_dev["b_qkv"], cs, q, k, v, scratch)
    torch.cuda.synchronize()
    return to_f64(q), to_f64(k), to_f64(v)


SMALL = W.LayerDims(256, 384, 4, 2)


@pytest.mark.parametrize("rule", ["key_norm_small", "window_attn"])
def test_layer_stack_full_retention_matches_oracle(rule, tile):
    """Three layers, three ragged groups, nothing pruned: every activation and every cache row must match."""
    print(f"case rule={rule}", flush=True)
    dims, frames, tpf, gf = SMALL, 10, 36, 4
    layers_t = [W.make_decoder_layer(dims, l) for l in range(3)]
    x = W.make_hidden(frames, tpf, dims.d_model)
    pos = W.video_positions(frames, tpf)
    x_win = torch.stack([W.make_hidden(1, 20, dims.d_model, seed=50 + l) for l in range(3)])
    pos_win = W.text_positions(20, frames)
    bounds = O.group_bounds(frames, tpf, gf)
    use_win = rule.startswith("window")
    got, caches, _ = _gpu_stack(dims, layers_t, x, pos, bounds, x_win if use_win else None, pos_win, rule, 1.0)
    want, want_caches = LO.layer_stack(to_f64(x), pos.numpy(), [oracle_weights(w, dims) for w in layers_t],
                                       oracle_shape(dims), bounds, to_f64(x_win) if use_win else None, pos_win.numpy(),
                                       rule, 1.0, store=LO.bf16_round)
    assert_layer_close(to_f64(got), want, "stack output", layers=3)
    for l, (cache, (ck, cv, cp)) in enumerate(zip(caches, want_caches)):
        assert cache.len == frames * tpf
        np.testing.assert_array_equal(cache.pos.cpu().numpy()[:, :cache.len], cp)
        assert_layer_close(to_f64(cache.k)[:, :cache.len], ck, f"layer {l} cached K", layers=l + 1)
        assert_layer_close(to_f64(cache.v)[:, :cache.len], cv, f"layer {l} cached V", layers=l + 1)


def test_layer_group_pruned_first_group_and_parts():
    """One group through one 7B-shaped layer at rho = 0.3: output, kept set, cache rows."""
    dims = W.LayerDims(3584, 18944, 28, 4)
    n_g = 300
    wt = W.make_decoder_layer(dims, 0)
    x = W.make_hidden(3, 100, dims.d_model)
    pos = W.video_positions(3, 100)
    got, caches, kept = _gpu_stack(dims, [wt], x, pos, [(0, n_g)], None, None, "key_norm_small", 0.3)
    shape = oracle_shape(dims)
    empty = np.zeros((dims.n_kv_heads, 0, 128))
    want, idx, nk, nv, mid = LO.layer_group(to_f64(x), pos.numpy(), oracle_weights(wt, dims), shape, empty, empty, None,
                                            "key_norm_small", 0.3, store=LO.bf16_round)
    assert_layer_close(to_f64(got), want, "layer output")
    # The selection is a function of the stored keys. The oracle's own keys differ from the GPU's by one-ulp flips in
    # a few elements, so the rule of the path applies to the keys the GPU stored: the oracle scores THOSE (widened
    # exactly) and its top-k must be the GPU's kept set, except between scores within 1e-5 (relative) of the k-th.
    got_idx = kept[0][2].cpu().numpy()
    wt_dev = {k_: v_.to(DEV) for k_, v_ in wt.items()}
    _, k_gpu, v_gpu = _gpu_group_qkv(dims, wt_dev, x.to(DEV), pos.to(DEV), 0, n_g)
    assert_layer_close(k_gpu, mid["k"], "rotated keys")
    scores_gpu_keys = O.score_kv("key_norm_small", k_gpu, v_gpu)
    excused = compare_kept(got_idx, O.topk_select(scores_gpu_keys, idx.shape[1]), scores_gpu_keys)
    print(f"kept sets on the GPU's stored keys: {excused} near-tie heads of {dims.n_kv_heads}", flush=True)
    for h in range(dims.n_kv_heads):
        # the appended rows are the GPU's own k, v at the kept tokens, bit for bit
        np.testing.assert_array_equal(to_f64(caches[0].k)[h, :90], k_gpu[got_idx[h], h])
        np.testing.assert_array_equal(to_f64(caches[0].v)[h, :90], v_gpu[got_idx[h], h])
        same = np.isin(got_idx[h], idx[h])
        assert same.mean() > 0.9                                 # against the oracle's own keys: nearly the same set
        rows = np.searchsorted(idx[h], got_idx[h][same])
        assert_layer_close(to_f64(caches[0].k)[h, :90][same], nk[h][rows], f"head {h} cached K")
        assert_layer_close(to_f64(caches[0].v)[h, :90][same], nv[h][rows], f"head {h} cached V")
    assert caches[0].len == 90


def test_layer_group_against_the_unrounded_definition():
    """The layer against the fp64 definition with NO rounding anywhere (store = identity). The kernels round to bf16
    where they store (h, q, k, v, attention output, x1, h2, the SwiGLU product, the output: 9 tensors on the way to
    an output element, each a relative error of at most 2^-9, independent in sign) and the attention rounds its
    softmax numerators (another 2^-9 per term): carried through the projections these add in quadrature to about
    sqrt(10) * 2^-9 / sqrt(3) = 3.6e-3 of the RMS. Gates: normalised error <= 1e-2 and every element within
    3e-2 |y| + 3e-2 rms (eight standard deviations). Nothing pruned, so no selection enters."""
    dims = SMALL
    n_g = 150
    wt = W.make_decoder_layer(dims, 2)
    x = W.make_hidden(6, 25, dims.d_model, seed=5)
    pos = W.video_positions(6, 25)
    got, caches, _ = _gpu_stack(dims, [wt], x, pos, [(0, n_g)], None, None, "value_norm", 1.0)
    empty = np.zeros((dims.n_kv_heads, 0, 128))
    want, _, nk, nv, _ = LO.layer_group(to_f64(x), pos.numpy(), oracle_weights(wt, dims), oracle_shape(dims), empty, empty,
                                        None, "value_norm", 1.0)
    got = to_f64(got)
    rms = np.sqrt(np.mean(want * want))
    err = np.abs(got - want)
    rel = np.linalg.norm(got - want) / np.linalg.norm(want)
    print(f"layer against the unrounded definition: normalised error {rel:.2e}, max abs {err.max():.2e}, rms {rms:.2e}",
          flush=True)
    assert np.isfinite(got).all() and rel <= 1e-2
    assert (err <= 3e-2 * np.abs(want) + 3e-2 * rms).all()
    for name, g_, w_ in (("K", to_f64(caches[0].k)[:, :n_g], nk), ("V", to_f64(caches[0].v)[:, :n_g], nv)):
        r = np.linalg.norm(g_ - w_) / np.linalg.norm(w_)
        print(f"cached {name} against the unrounded definition: normalised error {r:.2e}", flush=True)
        assert r <= 4e-3                                         # two roundings (h, then the projection's store)


def test_layer_group_full_size_sampled_rows():
    """The launch configuration bench.py times for the layer: config 2's group (2048 tokens) through a 7B-shaped layer,
    window-attention rule (64 window rows), against a pruned cache of 4920 entries per head. The oracle computes the
    normalised states, Q, K, V and the scores for all tokens, and everything that follows (attention, o_proj, MLP)
    for a sample of rows, one by one."""
    dims = W.LAYER_DIMS["7b"]
    w2 = W.CONFIGS["cfg2_7b_32k"]
    n_g, c, n_win = w2.group_tokens, 4920, w2.n_window
    hq, hkv, dm = dims.n_q_heads, dims.n_kv_heads, dims.d_model
    gen = torch.Generator().manual_seed(4242)
    wt = W.make_decoder_layer(dims, 3)
    x = W.make_hidden(w2.group_frames, w2.tokens_per_frame, dm, seed=11)
    pos = W.video_positions(w2.group_frames, w2.tokens_per_frame, first_frame=128)
    x_win = W.make_hidden(1, n_win, dm, seed=12)
    pos_win = W.text_positions(n_win, w2.n_frames)
    ck = torch.randn(hkv, c, 128, generator=gen).to(torch.bfloat16)
    cv = torch.randn(hkv, c, 128, generator=gen).to(torch.bfloat16)
    keep = B.keep_count(n_g, w2.retention)

    layout = B.make_layout(hq, hkv, 128, "bf16")
    shape = B.make_layer_shape(dm, dims.d_ff, dims.rms_eps, dims.rope_theta, dims.mrope_section)
    weights = B.LayerWeights(**{k_: v_.to(DEV) for k_, v_ in wt.items()})
    ws = B.make_layer_workspace(layout, shape, n_g, n_win)
    cache = B.Cache(layout, c + keep)
    cache.k[:, :c].copy_(ck)
    cache.v[:, :c].copy_(cv)
    cache.c.len = c
    q_win = torch.empty(n_win, hq, 128, dtype=torch.bfloat16, device=DEV)
    B.layer_window_queries(layout, shape, weights, x_win.to(DEV), pos_win.to(DEV), q_win, ws)
    out = torch.empty(n_g, dm, dtype=torch.bfloat16, device=DEV)
    kept = torch.empty(hkv, keep, dtype=torch.int32, device=DEV)
    B.layer_group(layout, shape, weights, x.to(DEV), pos.to(DEV), 0, 5000, q_win, "window_attn", keep, cache, out, kept, ws)
    torch.cuda.synchronize()
    assert cache.len == c + keep

    rb = LO.bf16_round
    ow, oshape = oracle_weights(wt, dims), oracle_shape(dims)
    x64 = to_f64(x)
    h = rb(LO.rms_norm(x64, ow["ln1"], dims.rms_eps))
    cos, sin = LO.mrope_cos_sin(pos.numpy(), 128, dims.rope_theta, dims.mrope_section)
    q = rb(LO.apply_rotary(LO.linear(h, ow["w_q"], ow["b_q"]).reshape(n_g, hq, 128), cos, sin))
    k = rb(LO.apply_rotary(LO.linear(h, ow["w_k"], ow["b_k"]).reshape(n_g, hkv, 128), cos, sin))
    v = rb(LO.linear(h, ow["w_v"], ow["b_v"]).reshape(n_g, hkv, 128))
    qw = LO.window_queries(to_f64(x_win), pos_win.numpy(), ow, oshape, store=rb)
    np.testing.assert_allclose(to_f64(q_win), qw, atol=2.0 ** -7 * np.abs(qw).max())     # one ulp at the largest value
    # selection: the oracle scores the keys and window queries the GPU stored (widened exactly); 1e-5 near-tie rule
    wt_dev = {k_: v_.to(DEV) for k_, v_ in wt.items()}
    _, k_gpu, v_gpu = _gpu_group_qkv(dims, wt_dev, x.to(DEV), pos.to(DEV), 0, n_g)
    assert_layer_close(k_gpu, k, "rotated keys")
    assert_layer_close(v_gpu, v, "values")
    scores = O.score_kv("window_attn", k_gpu, v_gpu, to_f64(q_win))
    got_idx = kept.cpu().numpy()
    excused = compare_kept(got_idx, O.topk_select(scores, keep), scores)
    print(f"kept sets on the GPU's stored keys: {excused} near-tie heads of {hkv}", flush=True)
    idx = O.topk_select(O.score_kv("window_attn", k, v, qw), keep)               # on the oracle's own keys
    for hh in range(hkv):
        np.testing.assert_array_equal(cache.pos.cpu().numpy()[hh, c:c + keep], 5000 + got_idx[hh])
        np.testing.assert_array_equal(to_f64(cache.k)[hh, c:c + keep], k_gpu[got_idx[hh], hh])
        np.testing.assert_array_equal(to_f64(cache.v)[hh, c:c + keep], v_gpu[got_idx[hh], hh])
        assert np.isin(got_idx[hh], idx[hh]).mean() > 0.9
    rows = sorted({0, 1, 127, 128, 255, 256, 1023, 1024, n_g - 129, n_g - 1} | set(np.random.default_rng(5).integers(0, n_g, 54).tolist()))
    a = rb(O.attend_group(q, k, v, to_f64(ck), to_f64(cv), rows=rows))                      # [len(rows), H_q, d]
    x1 = rb(x64[rows] + LO.linear(a.reshape(len(rows), hq * 128), ow["w_o"]))
    h2 = rb(LO.rms_norm(x1, ow["ln2"], dims.rms_eps))
    want = rb(x1 + LO.swiglu_mlp(h2, ow["w_gate"], ow["w_up"], ow["w_down"], store=rb))
    assert_layer_close(to_f64(out)[rows], want, "layer output, sampled rows")


def test_layer_text_chunk_and_decode_steps_after_video():
    """Sec. 2.1's later stages through the same layer call: after a video group, a chunk of text tokens and then
    single tokens (n_group_tokens = 7, then 1, nothing pruned) attend to everything cached so far. Two layers, so
    that the second layer's inputs are the first one's outputs at every step."""
    dims = SMALL
    layers_t = [W.make_decoder_layer(dims, l, seed=99) for l in range(2)]
    steps = [(0, 150), (150, 7), (157, 1), (158, 1), (159, 1)]
    n_tok = 160
    x = W.make_hidden(10, 16, dims.d_model, seed=5)
    pos = torch.cat([W.video_positions(10, 15)[:, :150], W.text_positions(10, 40)], dim=1).contiguous()
    got, caches, _ = _gpu_stack(dims, layers_t, x, pos, steps, None, None, "value_norm", 1.0)
    want, want_caches = LO.layer_stack(to_f64(x), pos.numpy(), [oracle_weights(w_, dims) for w_ in layers_t],
                                       oracle_shape(dims), steps, None, None, "value_norm", 1.0, store=LO.bf16_round)
    for base, n in steps:
        assert_layer_close(to_f64(got)[base:base + n], want[base:base + n], f"tokens {base}..{base + n - 1}", layers=2)
    for l, (cache, (ck, cv, cp)) in enumerate(zip(caches, want_caches)):
        assert cache.len == n_tok
        np.testing.assert_array_equal(cache.pos.cpu().numpy()[:, :n_tok], cp)
        assert_layer_close(to_f64(cache.k)[:, :n_tok], ck, f"layer {l} cached K", layers=l + 1)


@pytest.mark.parametrize("n_t", [1, 2])
@pytest.mark.parametrize("dims", [SMALL, W.LayerDims(3584, 18944, 28, 4)], ids=["small", "7b"])
def test_decode_step_equals_its_parts_bit_for_bit(dims, n_t):
    """One or two tokens through the layer: the projections stream their weights, and every token is kept, so the
    compaction is a plain append. The result must be, bit for bit, what the separate calls give: RMSNorm, rotary table, QKV, attention over the cache, o_proj + residual, RMSNorm, SwiGLU,
    down + residual; and the appended cache rows are the step's own K and V."""
    c0 = 333
    layout = B.make_layout(dims.n_q_heads, dims.n_kv_heads, 128, "bf16")
    shape = B.make_layer_shape(dims.d_model, dims.d_ff, dims.rms_eps, dims.rope_theta, dims.mrope_section)
    wt = {k_: v_.to(DEV) for k_, v_ in W.make_decoder_layer(dims, 0, seed=3).items()}
    weights = B.LayerWeights(**wt)
    g = torch.Generator(device=DEV).manual_seed(n_t)
    x = W.make_hidden(1, n_t, dims.d_model, seed=8).to(DEV)
    pos = W.text_positions(n_t, 900).to(DEV)
    ws = B.make_layer_workspace(layout, shape, n_t, 0)
    caches = []
    for _ in range(2):
        cache = B.Cache(layout, c0 + n_t)
        gg = torch.Generator(device=DEV).manual_seed(77)
        cache.k.copy_(torch.randn(cache.k.shape, generator=gg, device=DEV).bfloat16())
        cache.v.copy_(torch.randn(cache.v.shape, generator=gg, device=DEV).bfloat16())
        cache.c.len = c0
        caches.append(cache)
    # the layer call
    out = torch.full_like(x, float("nan"))
    kept = torch.full((dims.n_kv_heads, n_t), -1, dtype=torch.int32, device=DEV)
    B.layer_group(layout, shape, weights, x, pos, 0, 5000, None, "key_norm_small", n_t, caches[0], out, kept, ws)
    # the same step from its parts
    h = torch.empty_like(x)
    cs = torch.empty(n_t, 64, 2, dtype=torch.float32, device=DEV)
    q = torch.empty(n_t, dims.n_q_heads, 128, dtype=torch.bfloat16, device=DEV)
    k = torch.empty(n_t, dims.n_kv_heads, 128, dtype=torch.bfloat16, device=DEV)
    v = torch.empty_like(k)
    attn = torch.empty_like(q)
    x1, act, x2 = torch.empty_like(x), torch.empty(n_t, dims.d_ff, dtype=torch.bfloat16, device=DEV), torch.empty_like(x)
    split = torch.empty(32 << 20, dtype=torch.uint8, device=DEV)      # what the layer offers the attention
    B.rms_norm(x, wt["ln1_w"], h, dims.rms_eps)
    B.rope_table(pos, 0, n_t, dims.rope_theta, dims.mrope_section, cs)
    B.qkv_rope(layout, h, wt["w_qkv"], wt["b_qkv"], cs, q, k, v)
    B.group_attend(layout, q, k, v, caches[1], attn, None, split)
    B.linear(attn.view(n_t, -1), wt["w_o"], None, x, x1)
    B.rms_norm(x1, wt["ln2_w"], h, dims.rms_eps)
    B.swiglu_gate_up(h, wt["w_gate_up"], act)
    B.linear(act, wt["w_down"], None, x1, x2)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    assert torch.equal(out, x2)
    assert caches[0].len == c0 + n_t
    for h_ in range(dims.n_kv_heads):
        assert torch.equal(caches[0].k[h_, c0:c0 + n_t], k[:, h_]) and torch.equal(caches[0].v[h_, c0:c0 + n_t], v[:, h_])
        assert torch.equal(caches[0].k[h_, :c0], caches[1].k[h_, :c0])
    np.testing.assert_array_equal(kept.cpu().numpy(), np.tile(np.arange(n_t), (dims.n_kv_heads, 1)))
    np.testing.assert_array_equal(caches[0].pos.cpu().numpy()[:, c0:c0 + n_t], 5000 + np.tile(np.arange(n_t), (dims.n_kv_heads, 1)))


def test_layer_stack_replays_from_a_hip_graph():
    """A caller may capture the layer calls (side-stream fork/join, split projections and their second launches
    included) into a HIP graph: every replay, with eager work and synchronisations in between, reproduces the eager
    run bit for bit. Two layers, a video group, a short text chunk and a single token."""
    dims = SMALL
    layers_t = [W.make_decoder_layer(dims, l, seed=7) for l in range(2)]
    steps = [(0, 300), (300, 9), (309, 1)]
    x = W.make_hidden(20, 16, dims.d_model, seed=3)[:310].contiguous().to(DEV)
    pos = torch.cat([W.video_positions(20, 15)[:, :300], W.text_positions(10, 50)], dim=1).contiguous().to(DEV)
    layout = B.make_layout(dims.n_q_heads, dims.n_kv_heads, 128, "bf16")
    shape = B.make_layer_shape(dims.d_model, dims.d_ff, dims.rms_eps, dims.rope_theta, dims.mrope_section)
    weights = [B.LayerWeights(**{k: v.to(DEV) for k, v in w_.items()}) for w_ in layers_t]
    ws = B.make_layer_workspace(layout, shape, 300, 0)
    keeps = [B.keep_count(300, 0.5), 9, 1]
    caches = [B.Cache(layout, sum(keeps)) for _ in weights]
    out = torch.zeros_like(x)
    tmp = torch.empty(300, dims.d_model, dtype=torch.bfloat16, device=DEV)

    def run():
        for c in caches:
            c.reset()
        for (base, n), keep in zip(steps, keeps):
            B.layer_group(layout, shape, weights[0], x[base:base + n], pos, base, base, None, "key_norm_small", keep,
                          caches[0], tmp[:n], None, ws)
            B.layer_group(layout, shape, weights[1], tmp[:n], pos, base, base, None, "key_norm_small", keep,
                          caches[1], out[base:base + n], None, ws)

    run()
    torch.cuda.synchronize()
    want = [out.clone()] + [t.clone() for c in caches for t in (c.k, c.v, c.pos)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for replay in range(3):
        out.zero_()
        for c in caches:
            c.k.zero_(), c.v.zero_(), c.pos.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [out] + [t for c in caches for t in (c.k, c.v, c.pos)]
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {replay}"
        run()                                                    # eager work between the replays
        torch.cuda.synchronize()
        for a, b in zip([out] + [t for c in caches for t in (c.k, c.v, c.pos)], want):
            assert torch.equal(a, b), f"eager after replay {replay}"
