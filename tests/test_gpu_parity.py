"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same seeded inputs."""
import math

import numpy as np
import pytest
import torch

from helpers import assert_attn_close, compare_kept, sample_rows
from oracle import qp_oracle as O
from paper_2505_16175_amd import binding as B
from paper_2505_16175_amd.workload import CONFIGS, make_layer, scaled, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _f64(t):
    return to_f64(t)


def _kernels_for(layout):
    """Attention kernels to cover for a layout: the scalar one always, the MFMA one when it applies."""
    ks = [B.QP_ATTEND_SCALAR]
    if layout.dtype == B.QP_BF16 and layout.head_dim == 128:
        ks.append(B.QP_ATTEND_MFMA)
    return ks


@pytest.fixture(autouse=True)
def _reset_kernel_choice():
    yield
    B.select_attend_kernel(B.QP_ATTEND_AUTO)


# --------------------------------------------------------------------------------------------- S1
@pytest.mark.parametrize("dtype,h_q,h_kv,d", [("f32", 4, 2, 64), ("bf16", 28, 4, 128), ("bf16", 16, 2, 128),
                                              ("bf16", 8, 8, 64), ("f32", 6, 2, 128)])
@pytest.mark.parametrize("n_g,c", [(1, 0), (37, 5), (130, 0), (300, 200), (257, 1031)])
def test_group_attend_matches_oracle(dtype, h_q, h_kv, d, n_g, c):
    """Several tiles and ragged tails in both the group and the cache; sharp logits."""
    print(f"case dtype={dtype} heads={h_q}/{h_kv} d={d} n_g={n_g} c={c}", flush=True)
    g = torch.Generator().manual_seed(1000 * n_g + c + h_q)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    mk = lambda *s: (torch.randn(*s, generator=g) * 1.0).to(tdt)
    q, k, v = mk(n_g, h_q, d), mk(n_g, h_kv, d), mk(n_g, h_kv, d)
    ck, cv = mk(h_kv, c + 7, d), mk(h_kv, c + 7, d)          # capacity > len: stride is the capacity
    want, want_lse = O.attend_group(_f64(q), _f64(k), _f64(v), _f64(ck)[:, :c], _f64(cv)[:, :c], return_lse=True)
    layout = B.make_layout(h_q, h_kv, d, dtype)
    cache = B.Cache(layout, c + 7)
    cache.k.copy_(ck)
    cache.v.copy_(cv)
    cache.c.len = c
    for kern in _kernels_for(layout):
        B.select_attend_kernel(kern)
        out = torch.full((n_g, h_q, d), float("nan"), dtype=tdt, device=DEV)
        lse = torch.full((h_q, n_g), float("nan"), dtype=torch.float32, device=DEV)
        B.group_attend(layout, q.to(DEV), k.to(DEV), v.to(DEV), cache if c > 0 else None, out, lse)
        torch.cuda.synchronize()
        assert_attn_close(_f64(out), want, dtype, f"kernel {kern}")
        # bf16 MFMA kernel: the denominator is summed over bf16-rounded numerators (relative 2^-9 each)
        np.testing.assert_allclose(_f64(lse), want_lse, rtol=2e-5, atol=2e-5 if dtype == "f32" else 2e-3)
        assert cache.len == c


@pytest.mark.gpu
@pytest.mark.parametrize("h_q,h_kv", [(28, 4), (64, 8), (6, 3)])
@pytest.mark.parametrize("n_g,c", [(1, 9840), (1, 257), (64, 9840), (64, 5000), (7, 1031), (200, 3000), (1, 100)])
def test_group_attend_key_split_matches_oracle(h_q, h_kv, n_g, c):
    """Text-token prefill and decode over the pruned cache (Sec. 2.1, stages 2 and 3): few rows against a long
    cache. With scratch the MFMA kernel splits the cache over key chunks and merges; the result must match the
    oracle and the unsplit launch, output and log-sum-exp alike."""
    print(f"case heads={h_q}/{h_kv} n_g={n_g} c={c}", flush=True)
    d = 128
    g = torch.Generator().manual_seed(31 * n_g + c + h_q)
    mk = lambda *s: torch.randn(*s, generator=g).to(torch.bfloat16)
    q, k, v = mk(n_g, h_q, d), mk(n_g, h_kv, d), mk(n_g, h_kv, d)
    ck, cv = mk(h_kv, c + 3, d), mk(h_kv, c + 3, d)
    want, want_lse = O.attend_group(_f64(q), _f64(k), _f64(v), _f64(ck)[:, :c], _f64(cv)[:, :c], return_lse=True)
    layout = B.make_layout(h_q, h_kv, d, "bf16")
    cache = B.Cache(layout, c + 3)
    cache.k.copy_(ck)
    cache.v.copy_(cv)
    cache.c.len = c
    ws = B.make_workspace(layout, max(n_g, 32), 0)
    plan = B.attend_plan(layout, n_g, c, ws.numel())
    assert plan["kernel"] == (B.QP_ATTEND_MFMA_DECODE if n_g * (h_q // h_kv) <= 32 else B.QP_ATTEND_MFMA)
    assert plan["key_chunks"] > 1 or c < 4 * 64                     # with scratch, a long cache is split
    outs = []
    for scratch in (ws, None):
        out = torch.full((n_g, h_q, d), float("nan"), dtype=torch.bfloat16, device=DEV)
        lse = torch.full((h_q, n_g), float("nan"), dtype=torch.float32, device=DEV)
        B.group_attend(layout, q.to(DEV), k.to(DEV), v.to(DEV), cache, out, lse, scratch)
        torch.cuda.synchronize()
        assert_attn_close(_f64(out), want, "bf16", "split" if scratch is not None else "unsplit")
        np.testing.assert_allclose(_f64(lse), want_lse, rtol=2e-5, atol=2e-3)
        outs.append(out.float().cpu())
    # the two launches round the softmax numerators against different reference maxima: bf16-level agreement
    assert (outs[0] - outs[1]).abs().max().item() <= 2e-2


@pytest.mark.gpu
@pytest.mark.parametrize("h_q,h_kv,n_g,c,fp8", [(28, 4, 2400, 2100, False), (64, 8, 1100, 2100, False),
                                                (16, 16, 4400, 2100, False), (28, 4, 8192, 24000, False),
                                                (28, 4, 4096, 24000, False), (28, 4, 2400, 2100, True),
                                                (28, 4, 2350, 4099, False)])
def test_group_attend_last_round_split(h_q, h_kv, n_g, c, fp8):
    """Launches of several rounds of workgroups whose last round is only partly filled: with scratch, the row blocks
    of that round (the group's earliest tokens) are split over key chunks and merged, the others are not. Rows at both
    ends of the split region, at its boundary and sampled elsewhere against the oracle; every row against the launch
    without scratch (no split) at bf16 level."""
    print(f"case heads={h_q}/{h_kv} n_g={n_g} c={c} fp8={fp8}", flush=True)
    d, r = 128, h_q // h_kv
    g = torch.Generator(device=DEV).manual_seed(n_g + c)
    mk = lambda *s: torch.randn(*s, generator=g, device=DEV).bfloat16()
    q, k, v = mk(n_g, h_q, d), mk(n_g, h_kv, d), mk(n_g, h_kv, d)
    layout = B.make_layout(h_q, h_kv, d, "bf16")
    cache = B.Cache(layout, c + 5, fmt=B.QP_CACHE_FP8_E4M3 if fp8 else B.QP_CACHE_SAME)
    if fp8:
        cache.k.copy_((2.0 * torch.randn(h_kv, c + 5, d, generator=g, device=DEV)).to(torch.float8_e4m3fn))
        cache.v.copy_((2.0 * torch.randn(h_kv, c + 5, d, generator=g, device=DEV)).to(torch.float8_e4m3fn))
        ck64, cv64 = (t.float().double().cpu().numpy()[:, :c] for t in (cache.k, cache.v))
    else:
        cache.k.copy_(mk(h_kv, c + 5, d))
        cache.v.copy_(mk(h_kv, c + 5, d))
        ck64, cv64 = _f64(cache.k)[:, :c], _f64(cache.v)[:, :c]
    cache.c.len = c
    ws = B.make_workspace(layout, n_g, 0)
    plan = B.attend_plan(layout, n_g, c, ws.numel())
    n_rb = -(-n_g * r // 256)
    assert plan["kernel"] == B.QP_ATTEND_MFMA and plan["key_chunks"] >= 2 and plan["mirrored_rows"] == 0
    assert 0 < plan["split_row_blocks"] < n_rb and n_rb * h_kv > 256
    assert (plan["key_chunks"] - 1) * plan["tiles_per_chunk"] < -(-c // 64) <= plan["key_chunks"] * plan["tiles_per_chunk"]
    t_split = plan["split_row_blocks"] * 256 // r                     # first token with an unsplit row
    rows = sorted(set([0, 1, 63, 64, t_split - 2, t_split - 1, t_split, t_split + 1, n_g - 2, n_g - 1]
                      + [int(x) for x in sample_rows(n_g, 24, np.random.default_rng(c))]
                      + [int(x) for x in sample_rows(t_split, 8, np.random.default_rng(n_g))]))
    rows = np.array([x for x in rows if 0 <= x < n_g])
    want, want_lse = O.attend_group(_f64(q), _f64(k), _f64(v), ck64, cv64, rows=rows, return_lse=True)
    outs = []
    for scratch in (ws, None):
        out = torch.full_like(q, float("nan"))
        lse = torch.full((h_q, n_g), float("nan"), dtype=torch.float32, device=DEV)
        B.group_attend(layout, q, k, v, cache, out, lse, scratch)
        torch.cuda.synchronize()
        assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
        assert_attn_close(_f64(out[rows]), want, "bf16", "last round split" if scratch is not None else "no scratch")
        np.testing.assert_allclose(_f64(lse)[:, rows], want_lse, rtol=2e-5, atol=2e-3)
        outs.append((out.float(), lse.clone()))
    assert (outs[0][0] - outs[1][0]).abs().max().item() <= 2e-2
    assert (outs[0][1] - outs[1][1]).abs().max().item() <= 2e-3
    # rows outside the split region do not depend on the scratch at all
    assert torch.equal(outs[0][0][t_split + 1:], outs[1][0][t_split + 1:])


@pytest.mark.gpu
def test_group_attend_key_split_at_the_chunk_limit():
    """One workgroup's worth of rows against 24566 cache entries: the large kernel splits into its maximum of 128
    chunks, and the merge kernel takes two batches per wavefront."""
    h_q, h_kv, d, n_g, c = 64, 1, 128, 2, 24566
    g = torch.Generator().manual_seed(99)
    mk = lambda *s: torch.randn(*s, generator=g).to(torch.bfloat16)
    q, k, v, ck, cv = mk(n_g, h_q, d), mk(n_g, h_kv, d), mk(n_g, h_kv, d), mk(h_kv, c, d), mk(h_kv, c, d)
    want, want_lse = O.attend_group(_f64(q), _f64(k), _f64(v), _f64(ck), _f64(cv), return_lse=True)
    layout = B.make_layout(h_q, h_kv, d, "bf16")
    cache = B.Cache(layout, c)
    cache.k.copy_(ck)
    cache.v.copy_(cv)
    cache.c.len = c
    ws = B.make_workspace(layout, 32, 0)
    plan = B.attend_plan(layout, n_g, c, ws.numel())
    assert plan["kernel"] == B.QP_ATTEND_MFMA and plan["key_chunks"] == 128
    out = torch.full((n_g, h_q, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((h_q, n_g), float("nan"), dtype=torch.float32, device=DEV)
    B.group_attend(layout, q.to(DEV), k.to(DEV), v.to(DEV), cache, out, lse, ws)
    torch.cuda.synchronize()
    assert_attn_close(_f64(out), want, "bf16", "128 chunks")
    np.testing.assert_allclose(_f64(lse), want_lse, rtol=2e-5, atol=2e-3)


@pytest.mark.gpu
@pytest.mark.parametrize("h_q,h_kv,n_g", [(28, 4, 1), (28, 4, 4), (64, 8, 3), (6, 3, 16), (4, 4, 32), (32, 1, 1)])
@pytest.mark.parametrize("c", [0, 1, 31, 32, 33, 127, 128, 129, 1000, 4097])
def test_decode_shaped_attend_matches_oracle(h_q, h_kv, n_g, c):
    """At most 32 stacked rows per KV head: the kernel whose wavefronts stream their own 32-key blocks. Block
    boundaries of the cache (31/32/33, 127/128/129), an empty cache, several new tokens (causal among themselves),
    one workgroup per head (no scratch) and many (scratch + merge)."""
    print(f"case heads={h_q}/{h_kv} n_g={n_g} c={c}", flush=True)
    d = 128
    g = torch.Generator().manual_seed(977 * n_g + c + h_q)
    mk = lambda *s: torch.randn(*s, generator=g).to(torch.bfloat16)
    q, k, v = mk(n_g, h_q, d), mk(n_g, h_kv, d), mk(n_g, h_kv, d)
    ck, cv = mk(h_kv, c + 2, d), mk(h_kv, c + 2, d)
    want, want_lse = O.attend_group(_f64(q), _f64(k), _f64(v), _f64(ck)[:, :c], _f64(cv)[:, :c], return_lse=True)
    layout = B.make_layout(h_q, h_kv, d, "bf16")
    cache = B.Cache(layout, c + 2)
    cache.k.copy_(ck)
    cache.v.copy_(cv)
    cache.c.len = c
    ws = B.make_workspace(layout, 32, 0)
    assert B.attend_plan(layout, n_g, c, ws.numel())["kernel"] == B.QP_ATTEND_MFMA_DECODE
    for scratch in (ws, None):
        out = torch.full((n_g, h_q, d), float("nan"), dtype=torch.bfloat16, device=DEV)
        lse = torch.full((h_q, n_g), float("nan"), dtype=torch.float32, device=DEV)
        B.group_attend(layout, q.to(DEV), k.to(DEV), v.to(DEV), cache if c > 0 else None, out, lse, scratch)
        torch.cuda.synchronize()
        assert_attn_close(_f64(out), want, "bf16", "with scratch" if scratch is not None else "one workgroup per head")
        np.testing.assert_allclose(_f64(lse), want_lse, rtol=2e-5, atol=2e-3)


# --------------------------------------------------------------------------------------------- S2
@pytest.mark.parametrize("dtype,h_kv,d", [("f32", 2, 64), ("bf16", 4, 128), ("bf16", 8, 64), ("f32", 3, 128)])
@pytest.mark.parametrize("n_g", [1, 33, 2048, 5000])
def test_norm_scores_match_oracle(dtype, h_kv, d, n_g):
    print(f"case dtype={dtype} h_kv={h_kv} d={d} n_g={n_g}", flush=True)
    g = torch.Generator().manual_seed(n_g + d)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    k = (torch.randn(n_g, h_kv, d, generator=g) * torch.exp(0.5 * torch.randn(n_g, 1, 1, generator=g))).to(tdt)
    v = torch.randn(n_g, h_kv, d, generator=g).to(tdt)
    k[0] = 0                                                   # a zero row: score +0.0 under both rules
    layout = B.make_layout(h_kv * 2, h_kv, d, dtype)
    for rule in ("key_norm_small", "value_norm"):
        s = torch.full((h_kv, n_g), float("nan"), dtype=torch.float32, device=DEV)
        B.score_kv(layout, rule, k.to(DEV), v.to(DEV), None, s)
        torch.cuda.synchronize()
        want = O.score_kv(rule, _f64(k), _f64(v))
        np.testing.assert_allclose(_f64(s), want, rtol=1e-6, atol=0)
    assert not np.signbit(_f64(s)[0, 0])


@pytest.mark.parametrize("dtype,h_q,h_kv,d,w", [("f32", 4, 2, 64, 16), ("bf16", 28, 4, 128, 64), ("bf16", 16, 2, 128, 128),
                                                ("bf16", 8, 8, 64, 5)])
@pytest.mark.parametrize("n_g,sharp", [(32, True), (300, True), (2048, False), (1000, True)])
def test_window_scores_match_oracle(dtype, h_q, h_kv, d, w, n_g, sharp):
    print(f"case dtype={dtype} heads={h_q}/{h_kv} d={d} w={w} n_g={n_g} sharp={sharp}", flush=True)
    g = torch.Generator().manual_seed(n_g + w)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    sc = 1.0 if sharp else 1.0 / math.sqrt(d)
    k = (torch.randn(n_g, h_kv, d, generator=g) * sc).to(tdt)
    qw = (torch.randn(w, h_q, d, generator=g) * sc).to(tdt)
    layout = B.make_layout(h_q, h_kv, d, dtype)
    ws = B.make_workspace(layout, n_g, w)
    s = torch.full((h_kv, n_g), float("nan"), dtype=torch.float32, device=DEV)
    B.score_kv(layout, "window_attn", k.to(DEV), None, qw.to(DEV), s, ws)
    torch.cuda.synchronize()
    want = O.score_kv("window_attn", _f64(k), None, _f64(qw))
    got = _f64(s)
    np.testing.assert_allclose(got, want, rtol=2e-5, atol=1e-7)
    np.testing.assert_allclose(got.sum(axis=1), (h_q // h_kv) * w, rtol=1e-5)   # total attention mass


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,h_q,h_kv,d,w", [("f32", 4, 2, 64, 16), ("bf16", 28, 4, 128, 64), ("bf16", 64, 8, 128, 128),
                                                ("f32", 6, 3, 128, 5)])
@pytest.mark.parametrize("n_g", [1, 33, 2048, 5000])
def test_window_logit_scores_match_oracle(dtype, h_q, h_kv, d, w, n_g):
    """The softmax-free variant of the attention-score rule (one dot product per key against the summed window)."""
    print(f"case dtype={dtype} heads={h_q}/{h_kv} d={d} w={w} n_g={n_g}", flush=True)
    g = torch.Generator().manual_seed(n_g + 13 * w)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    k = torch.randn(n_g, h_kv, d, generator=g).to(tdt)
    qw = torch.randn(w, h_q, d, generator=g).to(tdt)
    want = O.score_kv("window_logit", _f64(k), None, _f64(qw))
    layout = B.make_layout(h_q, h_kv, d, dtype)
    ws = B.make_workspace(layout, n_g, w)
    scores = torch.full((h_kv, n_g), float("nan"), dtype=torch.float32, device=DEV)
    B.score_kv(layout, "window_logit", k.to(DEV), None, qw.to(DEV), scores, ws)
    torch.cuda.synchronize()
    # f32 sums of (R*W) rows and of d products: relative to the size of the terms, not of the (cancelling) result
    bound = 2e-6 * np.abs(_f64(qw)).sum(axis=(0, 1)).max() * np.abs(_f64(k)).max() * d / math.sqrt(d)
    np.testing.assert_allclose(scores.cpu().numpy(), want, rtol=1e-5, atol=max(bound, 1e-6))


@pytest.mark.gpu
@pytest.mark.parametrize("rule", ["key_norm_small+shared", "window_attn+shared", "window_logit+shared"])
def test_head_shared_scores_and_selection(rule):
    """QP_SCORE_SHARED_HEADS: every head's score row becomes the f32 sum over heads (in head order), so the per-head
    TopK keeps one index set; checked bit-exactly against the same sum done by hand, and against the oracle."""
    h_q, h_kv, d, w, n_g, keep = 28, 4, 128, 64, 1500, 300
    g = torch.Generator().manual_seed(5)
    k = torch.randn(n_g, h_kv, d, generator=g).to(torch.bfloat16)
    v = torch.randn(n_g, h_kv, d, generator=g).to(torch.bfloat16)
    qw = torch.randn(w, h_q, d, generator=g).to(torch.bfloat16)
    layout = B.make_layout(h_q, h_kv, d, "bf16")
    ws = B.make_workspace(layout, n_g, w)
    base = torch.empty(h_kv, n_g, dtype=torch.float32, device=DEV)
    shared = torch.empty_like(base)
    B.score_kv(layout, rule.split("+")[0], k.to(DEV), v.to(DEV), qw.to(DEV), base, ws)
    B.score_kv(layout, rule, k.to(DEV), v.to(DEV), qw.to(DEV), shared, ws)
    torch.cuda.synchronize()
    by_hand = base[0].clone()
    for h in range(1, h_kv):
        by_hand += base[h]
    assert torch.equal(shared, by_hand.expand_as(shared))
    want = O.score_kv(rule, _f64(k), _f64(v), _f64(qw))
    np.testing.assert_allclose(shared.cpu().numpy(), want, rtol=2e-4, atol=2e-4)
    cache = B.Cache(layout, keep)
    kept = torch.empty(h_kv, keep, dtype=torch.int32, device=DEV)
    B.topk_compact(layout, shared, k.to(DEV), v.to(DEV), keep, 0, cache, kept)
    torch.cuda.synchronize()
    got = kept.cpu().numpy()
    assert (got == got[0]).all()                               # one index set for all heads
    np.testing.assert_array_equal(got, O.topk_select(shared.cpu().double().numpy(), keep))


# --------------------------------------------------------------------------------------------- S3 + S4
@pytest.mark.parametrize("dtype,h_kv,d", [("bf16", 4, 128), ("f32", 2, 64)])
@pytest.mark.parametrize("n_g,keep,ties", [(4, 2, True), (1, 1, False), (100, 100, True), (1000, 1, True),
                                           (2048, 615, False), (8192, 820, True), (5000, 4999, False),
                                           (32768, 20000, True), (32768, 3277, False)])
def test_topk_compact_exact(dtype, h_kv, d, n_g, keep, ties):
    """Same f32 scores on both sides: kept sets, positions and copied rows must be bit-exact."""
    print(f"case dtype={dtype} h_kv={h_kv} d={d} n_g={n_g} keep={keep} ties={ties}", flush=True)
    g = torch.Generator().manual_seed(n_g * 7 + keep)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    s = torch.randn(h_kv, n_g, generator=g)
    if ties:
        s = torch.round(s * 4) / 4                              # heavy ties, includes -0.0 and +0.0
        s[0, : n_g // 2] = 0.5                                  # a long run of equal scores
        if n_g >= 4:
            s[-1, :] = -1.25                                    # all equal: the first `keep` tokens survive
    k = torch.randn(n_g, h_kv, d, generator=g).to(tdt)
    v = torch.randn(n_g, h_kv, d, generator=g).to(tdt)
    layout = B.make_layout(h_kv, h_kv, d, dtype)
    pre, base = 3, 77000
    cache = B.Cache(layout, pre + keep + 5)
    cache.c.len = pre
    kept = torch.full((h_kv, keep), -1, dtype=torch.int32, device=DEV)
    B.topk_compact(layout, s.to(DEV), k.to(DEV), v.to(DEV), keep, base, cache, kept)
    torch.cuda.synchronize()
    assert cache.len == pre + keep
    want = O.topk_select(s.double().numpy(), keep)
    got = kept.cpu().numpy()
    np.testing.assert_array_equal(got, want)
    if ties and n_g >= 4:
        assert got[-1].tolist() == list(range(keep))
    pos = cache.pos.cpu().numpy()
    np.testing.assert_array_equal(pos[:, pre:pre + keep], base + want)
    assert (pos[:, :pre] == -1).all() and (pos[:, pre + keep:] == -1).all()       # nothing else written
    ck, cv = cache.k.cpu(), cache.v.cpu()
    for h in range(h_kv):
        idx = torch.from_numpy(want[h])
        assert torch.equal(ck[h, pre:pre + keep], k[idx, h]) and torch.equal(cv[h, pre:pre + keep], v[idx, h])
        assert (ck[h, :pre] == 0).all() and (ck[h, pre + keep:] == 0).all()


@pytest.mark.parametrize("h_kv,n_g,keep", [(70, 2048, 615), (300, 513, 77), (112, 8192, 820)])
def test_topk_compact_many_heads(h_kv, n_g, keep):
    """Many KV heads (the bandwidth-characterisation shape of bench.py folds layers into heads): the slices per head
    are capped by the head count, down to one workgroup per head; kept sets, positions and rows stay bit-exact."""
    print(f"case h_kv={h_kv} n_g={n_g} keep={keep}", flush=True)
    g = torch.Generator().manual_seed(h_kv + n_g)
    s = torch.round(torch.randn(h_kv, n_g, generator=g) * 64) / 64          # some ties
    k = torch.randn(n_g, h_kv, 128, generator=g).to(torch.bfloat16)
    v = torch.randn(n_g, h_kv, 128, generator=g).to(torch.bfloat16)
    layout = B.make_layout(h_kv, h_kv, 128, "bf16")
    cache = B.Cache(layout, keep + 2)
    cache.c.len = 2
    B.topk_compact(layout, s.to(DEV), k.to(DEV), v.to(DEV), keep, 1000, cache, None)
    torch.cuda.synchronize()
    want = O.topk_select(s.double().numpy(), keep)
    np.testing.assert_array_equal(cache.pos.cpu().numpy()[:, 2:2 + keep], 1000 + want)
    ck, cv = cache.k.cpu(), cache.v.cpu()
    for h in range(0, h_kv, 7):
        idx = torch.from_numpy(want[h])
        assert torch.equal(ck[h, 2:2 + keep], k[idx, h]) and torch.equal(cv[h, 2:2 + keep], v[idx, h])
        assert (ck[h, :2] == 0).all()


def _score_families(n_g, g):
    """Score vectors that drive the selection through each of its routes (one KV head per family)."""
    base = torch.rand(n_g, generator=g)
    fams = {}
    # adjacent floats: the whole key range is narrower than one round of buckets
    fams["adjacent"] = torch.from_numpy(
        (np.float32(1.0).view(np.int32) + torch.randint(0, 1500, (n_g,), generator=g).numpy().astype(np.int32))
        .view(np.float32).copy())
    # two far outliers stretch the range so that nearly all keys share a bucket: needs further rounds
    dense = 3.0 + base * 1e-3
    dense[n_g // 3] = 1e30
    dense[n_g // 2] = -1e30
    fams["dense_with_outliers"] = dense
    # both signs, both zeros, and far more ties at the threshold than the direct-ranking list holds
    mixed = torch.where(base < 0.2, torch.tensor(-2.5), torch.where(base < 0.7, torch.tensor(0.0), torch.tensor(7.0)))
    mixed[::5] = -0.0
    fams["signs_and_zeros"] = mixed
    # infinities at both ends and a log-uniform body over 60 octaves
    wide = torch.exp2((base - 0.5) * 60.0) * torch.where(torch.rand(n_g, generator=g) < 0.5, -1.0, 1.0)
    wide[0], wide[n_g - 1] = float("inf"), float("-inf")
    fams["wide_with_inf"] = wide
    return fams


@pytest.mark.gpu
@pytest.mark.parametrize("n_g", [700, 2048, 8192, 32768])
@pytest.mark.parametrize("keep_frac", [0.0, 0.1, 0.5, 1.0])
def test_topk_select_routes(n_g, keep_frac):
    """Eq. 2's TopK on score distributions chosen for the selection's branches (exact bucket, repeated rounds,
    direct ranking, ties beyond the list): kept indices are bit-exact against the oracle's stable selection."""
    keep = min(n_g, max(1, int(round(keep_frac * n_g))))
    print(f"case n_g={n_g} keep={keep}", flush=True)
    g = torch.Generator().manual_seed(n_g + keep)
    fams = _score_families(n_g, g)
    s = torch.stack(list(fams.values())).float().contiguous()
    h_kv, d = s.shape[0], 64
    k = torch.randn(n_g, h_kv, d, generator=g)
    v = torch.randn(n_g, h_kv, d, generator=g)
    layout = B.make_layout(h_kv, h_kv, d, "f32")
    cache = B.Cache(layout, keep)
    kept = torch.full((h_kv, keep), -1, dtype=torch.int32, device=DEV)
    B.topk_compact(layout, s.to(DEV), k.to(DEV), v.to(DEV), keep, 0, cache, kept)
    torch.cuda.synchronize()
    want = O.topk_select(s.double().numpy(), keep)
    got = kept.cpu().numpy()
    for h, name in enumerate(fams):
        np.testing.assert_array_equal(got[h], want[h], err_msg=name)
    np.testing.assert_array_equal(cache.pos.cpu().numpy()[:, :keep], want)
    ck = cache.k.cpu()
    for h in range(h_kv):
        assert torch.equal(ck[h, :keep], k[torch.from_numpy(want[h]), h])


# --------------------------------------------------------------------------------------------- whole path
def _run_prefill(w, q, k, v, qw, rule, kernel=B.QP_ATTEND_AUTO):
    layout = B.make_layout(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
    cap = B.cache_capacity(w.n_frames, w.tokens_per_frame, w.group_frames, w.retention)
    cache = B.Cache(layout, cap)
    ws = B.make_workspace(layout, min(w.group_tokens, w.n_tokens), w.n_window if rule.startswith("window") else 0)
    out = torch.full_like(q, float("nan"))
    B.select_attend_kernel(kernel)
    B.prefill_video(layout, w.n_frames, w.tokens_per_frame, w.group_frames, w.retention, rule, q, k, v,
                    qw if rule.startswith("window") else None, cache, out, ws)
    torch.cuda.synchronize()
    return out, cache


def _check_cache_against_oracle(w, k, v, qw, rule, cache):
    """Kept sets of every group vs the oracle (near-ties counted), and the compaction as a bit-exact copy.

    Returns (sel, pos, near, sel_valid). sel is the oracle's own selection. sel_valid is the same list with
    the kept indices of the (group, head) pairs that differ by an excused near-tie replaced by the GPU's:
    equal-within-1e-5 scores admit more than one correct kept set, the attention of later groups is
    unique only once that choice is fixed, and the GPU's choice has just been validated against the
    oracle's scores. The cache the oracle attends over is always gathered on the host from the inputs.
    """
    k64, v64 = _f64(k), _f64(v)
    sel = O.select_all_groups(k64, v64, None if qw is None else _f64(qw), w.n_frames, w.tokens_per_frame,
                              w.group_frames, w.retention, rule)
    assert cache.len == sum(i.shape[1] for _, _, i, _ in sel) == O.final_cache_len(
        w.n_frames, w.tokens_per_frame, w.group_frames, w.retention)
    pos = cache.pos.cpu().numpy()[:, :cache.len]
    lo, near = 0, 0
    sel_valid = []
    for base, n_g, idx, s in sel:
        kk = idx.shape[1]
        got = pos[:, lo:lo + kk] - base
        near += compare_kept(got, idx, s)
        sel_valid.append((base, n_g, got.astype(np.int64), s))
        lo += kk
    ck, cv = cache.k.cpu(), cache.v.cpu()
    kc, vc = k.cpu(), v.cpu()
    for h in range(w.n_kv_heads):
        p = torch.from_numpy(pos[h].astype(np.int64))
        assert torch.equal(ck[h, :cache.len], kc[p, h]) and torch.equal(cv[h, :cache.len], vc[p, h])
    return sel, pos, near, sel_valid


def _oracle_outputs(w, q, k, v, sel_valid):
    """The oracle's attention of every group over the cache fixed by sel_valid (group by group)."""
    q64, k64, v64 = _f64(q), _f64(k), _f64(v)
    out = np.zeros_like(q64)
    for gi, (base, n_g, _, _) in enumerate(sel_valid):
        ck, cv, _ = O.gather_cache(k64, v64, sel_valid, gi)
        sl = slice(base, base + n_g)
        out[sl] = O.attend_group(q64[sl], k64[sl], v64[sl], ck, cv)
    return out


@pytest.mark.parametrize("sharp", [False, True])
@pytest.mark.parametrize("rule", ["key_norm_small", "window_attn", "value_norm"])
def test_cfg1_tiny_whole_path(rule, sharp):
    w = CONFIGS["cfg1_tiny_f32"]
    print(f"case cfg1 rule={rule} sharp={sharp}", flush=True)
    q, k, v, qw = make_layer(w, sharp=sharp)
    want, wck, wcv, wpos, _ = O.prefill_video(_f64(q), _f64(k), _f64(v), _f64(qw), w.n_frames, w.tokens_per_frame,
                                              w.group_frames, w.retention, rule)
    out, cache = _run_prefill(w, q.to(DEV), k.to(DEV), v.to(DEV), qw.to(DEV), rule)
    _, pos, near, sel_valid = _check_cache_against_oracle(w, k, v, qw, rule, cache)
    assert cache.len == 64
    if near == 0:
        np.testing.assert_array_equal(pos, wpos)
    else:
        want = _oracle_outputs(w, q, k, v, sel_valid)
    assert_attn_close(_f64(out), want, "f32", "cfg1")


@pytest.mark.parametrize("name,frames,tokens_per_frame,group_frames", [
    ("cfg2_7b_32k", 12, 40, 5),          # ragged: last group 2 frames, group tokens 200 (not a tile multiple)
    ("cfg4_72b_128k", 6, 96, 2),
    ("cfg3_7b_128k_norm", 9, 64, 4),
    ("cfg2_7b_32k", 40, 32, 1),          # one-frame groups against a growing cache: the attention's key split
    ("cfg4_72b_128k", 30, 64, 1),        # engages on both attention streams of the call
])
@pytest.mark.parametrize("sharp", [False, True])
def test_reduced_configs_whole_path_full_oracle(name, frames, tokens_per_frame, group_frames, sharp):
    """The benchmark layer shapes at reduced length: every output element against the full oracle."""
    w = scaled(CONFIGS[name], n_frames=frames, tokens_per_frame=tokens_per_frame, group_frames=group_frames)
    for rule in w.rules:
        q, k, v, qw = make_layer(w, sharp=sharp)
        want, *_ = O.prefill_video(_f64(q), _f64(k), _f64(v), None if qw is None else _f64(qw), w.n_frames,
                                   w.tokens_per_frame, w.group_frames, w.retention, rule)
        dq, dk, dv = q.to(DEV), k.to(DEV), v.to(DEV)
        dqw = None if qw is None else qw.to(DEV)
        layout = B.make_layout(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
        for kern in _kernels_for(layout):
            print(f"case {name} reduced rule={rule} sharp={sharp} kernel={kern}", flush=True)
            out, cache = _run_prefill(w, dq, dk, dv, dqw, rule, kern)
            _, _, near, sel_valid = _check_cache_against_oracle(w, k, v, qw, rule, cache)
            # a near-tie changes the cache, hence later outputs: then the oracle attends over the validated choice
            ref = want if near == 0 else _oracle_outputs(w, q, k, v, sel_valid)
            assert_attn_close(_f64(out), ref, w.dtype, f"{name} kernel {kern}")


@pytest.mark.parametrize("rule", ["window_logit", "key_norm_small+shared", "window_attn+shared"])
def test_rule_variants_whole_path(rule):
    """The rule variants through qp_prefill_video on a reduced config-2 shape, every output element against the oracle."""
    w = scaled(CONFIGS["cfg2_7b_32k"], n_frames=12, tokens_per_frame=40, group_frames=5)
    q, k, v, qw = make_layer(w, sharp=True)
    dq, dk, dv, dqw = q.to(DEV), k.to(DEV), v.to(DEV), qw.to(DEV)
    out, cache = _run_prefill(w, dq, dk, dv, dqw, rule)
    _, _, near, sel_valid = _check_cache_against_oracle(w, k, v, qw, rule, cache)
    if rule.endswith("+shared"):
        pos = cache.pos.cpu().numpy()[:, :cache.len]
        assert (pos == pos[0]).all()
    assert_attn_close(_f64(out), _oracle_outputs(w, q, k, v, sel_valid), w.dtype, rule)


def _full_size_check(w, rule, sharp, n_rows, layer=0, whole_groups=(), sample_groups=None):
    """Full-size run in the launch configuration bench.py times: the whole output finite (it is pre-filled with NaN,
    so a workgroup that wrote nothing shows), kept sets of all groups and the cache copy against the oracle, sampled
    attention rows in `sample_groups` (default: first, second, middle, last) and every row of `whole_groups`."""
    q, k, v, qw = make_layer(w, layer=layer, device=DEV, sharp=sharp)
    out, cache = _run_prefill(w, q, k, v, qw, rule)
    assert bool(torch.isfinite(out).all()), f"{w.name}: rows of the output were not written"
    sel, pos, near, sel_valid = _check_cache_against_oracle(w, k, v, qw, rule, cache)
    rng = np.random.default_rng(5)
    bounds = B.group_bounds(w.n_frames, w.tokens_per_frame, w.group_frames)
    assert bounds == [tuple(b) for b in O.group_bounds(w.n_frames, w.tokens_per_frame, w.group_frames)]
    groups = sorted({0, 1, len(bounds) // 2, len(bounds) - 1}) if sample_groups is None else list(sample_groups)
    k64, v64 = _f64(k), _f64(v)
    stats = []
    for gi in sorted(set(groups) | set(whole_groups)):
        base, n_g = bounds[gi]
        rows = None if gi in whole_groups else sample_rows(n_g, n_rows, rng)
        sl = slice(base, base + n_g)
        ck, cv, _ = O.gather_cache(k64, v64, sel_valid, gi)    # gathered on the host from the inputs
        want = O.attend_group(_f64(q[sl]), k64[sl], v64[sl], ck, cv, rows=rows)
        got = _f64(out[sl]) if rows is None else _f64(out[sl][rows])
        stats.append(assert_attn_close(got, want, w.dtype, f"{w.name} group {gi}"))
    return near, stats, cache


def test_cfg2_full_size():
    w = CONFIGS["cfg2_7b_32k"]
    for sharp in (False, True):
        print(f"case cfg2 full size sharp={sharp}", flush=True)
        # first and last group element by element (every row of 2048 x 28 heads), sampled rows in two more
        near, stats, cache = _full_size_check(w, "window_attn", sharp, 24, whole_groups=(0, 15))
        print(f"  near-tie heads excused: {near}; max abs err {max(s['max_abs'] for s in stats):.3e}; "
              f"max normalised err {max(s['nrm'] for s in stats):.3e}", flush=True)
        assert cache.len == 9840


@pytest.mark.parametrize("rule", ["key_norm_small", "value_norm"])
def test_cfg3_full_size(rule):
    w = CONFIGS["cfg3_7b_128k_norm"]
    print(f"case cfg3 full size rule={rule}", flush=True)
    near, stats, cache = _full_size_check(w, rule, False, 16)
    print(f"  near-tie heads excused: {near}; max abs err {max(s['max_abs'] for s in stats):.3e}; "
          f"max normalised err {max(s['nrm'] for s in stats):.3e}", flush=True)
    assert cache.len == 26240


@pytest.mark.parametrize("sharp", [False, True])
def test_cfg4_full_size(sharp):
    w = CONFIGS["cfg4_72b_128k"]
    print(f"case cfg4 full size sharp={sharp}", flush=True)
    near, stats, cache = _full_size_check(w, "window_attn", sharp, 16)
    print(f"  near-tie heads excused: {near}; max abs err {max(s['max_abs'] for s in stats):.3e}; "
          f"max normalised err {max(s['nrm'] for s in stats):.3e}", flush=True)
    assert cache.len == 32768


@pytest.mark.parametrize("layer", [0, 13, 27])
def test_cfg5_full_size_layer(layer):
    """One layer of the hour-long stack at full size (ragged last group of 16 frames); layers are independent."""
    w = CONFIGS["cfg5_7b_hour_stack"]
    print(f"case cfg5 full size layer={layer}", flush=True)
    near, stats, cache = _full_size_check(w, "window_attn", False, 12, layer=layer)
    print(f"  near-tie heads excused: {near}; max abs err {max(s['max_abs'] for s in stats):.3e}; "
          f"max normalised err {max(s['nrm'] for s in stats):.3e}", flush=True)
    assert cache.len == 46125
    # resident pruned cache of one layer: 2 * H_kv * len * d * 2 bytes (the KV-cache memory equation of App. D.2 times rho)
    assert cache.nbytes() == 2 * 4 * 46125 * 128 * 2
    want = O.kv_cache_bytes(1, w.n_tokens, w.n_kv_heads, w.head_dim, 2, retention=cache.len / w.n_tokens)
    assert abs(cache.nbytes() - want) < 1e-6 * want


@pytest.mark.parametrize("first_layer", [0, 7, 14, 21])
def test_cfg5_every_layer_kept_sets_and_cache(first_layer):
    """All 28 layers of the hour-long stack (seven per case): the kept set of every group and head against the
    oracle, and the pruned cache as a bit-exact copy of the kept rows. Scores depend on a group's own K, V and the
    window only (Eq. 2 writes s(K_g, V_g)), so the oracle needs no attention for this. The stack's resident cache is
    28 times one layer's."""
    w = CONFIGS["cfg5_7b_hour_stack"]
    total_near = 0
    for layer in range(first_layer, first_layer + 7):
        q, k, v, qw = make_layer(w, layer=layer, device=DEV)
        out, cache = _run_prefill(w, q, k, v, qw, "window_attn")
        assert bool(torch.isfinite(out).all())
        _, _, near, _ = _check_cache_against_oracle(w, k, v, qw, "window_attn", cache)
        assert cache.len == 46125 and cache.nbytes() == 2 * 4 * 46125 * 128 * 2
        total_near += near
        print(f"cfg5 layer {layer}: kept sets and cache rows match; near-tie heads excused {near}", flush=True)
        del q, k, v, qw, out, cache
    assert 28 * 2 * 4 * 46125 * 128 * 2 == 2644992000              # 2.645 GB resident for the stack
    print(f"cfg5 layers {first_layer}..{first_layer + 6}: near-tie heads excused in total {total_near}", flush=True)


# --------------------------------------------------------------------------------------------- behaviour of the boundary
def test_runs_are_deterministic_and_stream_ordered():
    """Same inputs twice -> bit-identical cache, positions and outputs; a non-default caller stream is honoured."""
    w = scaled(CONFIGS["cfg2_7b_32k"], n_frames=24, tokens_per_frame=96, group_frames=5)
    q, k, v, qw = make_layer(w, device=DEV, sharp=True)
    results = []
    side = torch.cuda.Stream()
    for use_side in (False, True, False):
        if use_side:
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                out, cache = _run_prefill(w, q, k, v, qw, "window_attn")
                # work enqueued on the caller's stream after the call sees all of its results, without a host sync
                snap = (out.clone(), cache.k.clone(), cache.v.clone(), cache.pos.clone())
            torch.cuda.current_stream().wait_stream(side)
        else:
            out, cache = _run_prefill(w, q, k, v, qw, "window_attn")
            snap = (out.clone(), cache.k.clone(), cache.v.clone(), cache.pos.clone())
        torch.cuda.synchronize()
        results.append(snap)
    for other in results[1:]:
        for a, b in zip(results[0], other):
            assert torch.equal(a, b)


def test_prefill_can_be_resumed_from_the_cache():
    """The pruned cache and its length are the whole state between groups (Sec. 3.2: the kept KV is what is stored):
    a layer prefilled for the first groups by qp_prefill_video and continued group by group with the three step calls
    (the cache's len carrying on, positions offset by the tokens already seen) ends bit-identical to one
    qp_prefill_video over the whole video."""
    w = scaled(CONFIGS["cfg2_7b_32k"], n_frames=23, tokens_per_frame=64, group_frames=4)   # 5 groups + a short one
    q, k, v, qw = make_layer(w, device=DEV, sharp=True)
    want_out, want_cache = _run_prefill(w, q, k, v, qw, "window_attn")
    layout = B.make_layout(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
    cache = B.Cache(layout, B.cache_capacity(w.n_frames, w.tokens_per_frame, w.group_frames, w.retention))
    ws = B.make_workspace(layout, w.group_tokens, w.n_window)
    out = torch.full_like(q, float("nan"))
    head_frames = 3 * w.group_frames
    n_head = head_frames * w.tokens_per_frame
    B.prefill_video(layout, head_frames, w.tokens_per_frame, w.group_frames, w.retention, "window_attn",
                    q[:n_head], k[:n_head], v[:n_head], qw, cache, out[:n_head], ws)
    torch.cuda.synchronize()
    assert cache.len == 3 * B.keep_count(w.group_tokens, w.retention)
    for base, n_g in B.group_bounds(w.n_frames, w.tokens_per_frame, w.group_frames)[3:]:              # two full groups and the short last one
        sl = slice(base, base + n_g)
        scores = torch.empty(w.n_kv_heads, n_g, dtype=torch.float32, device=DEV)
        B.group_attend(layout, q[sl], k[sl], v[sl], cache, out[sl], None, ws)
        B.score_kv(layout, "window_attn", k[sl], v[sl], qw, scores, ws)
        B.topk_compact(layout, scores, k[sl], v[sl], B.keep_count(n_g, w.retention), base, cache, None, ws)
    torch.cuda.synchronize()
    assert cache.len == want_cache.len
    assert torch.equal(out, want_out)
    n = cache.len
    assert torch.equal(cache.k[:, :n], want_cache.k[:, :n]) and torch.equal(cache.v[:, :n], want_cache.v[:, :n])
    assert torch.equal(cache.pos[:, :n], want_cache.pos[:, :n])


@pytest.mark.parametrize("group_frames", [5, 1])
def test_prefill_video_replays_from_a_hip_graph(group_frames):
    """A caller may capture qp_prefill_video (its forked library streams included) into a HIP graph: every replay,
    with eager work and synchronisations in between, reproduces the eager call bit for bit. One-frame groups make
    the attention launches take the key split (two launches and scratch per group) inside the graph."""
    w = scaled(CONFIGS["cfg2_7b_32k"], n_frames=24, tokens_per_frame=64, group_frames=group_frames)
    q, k, v, qw = make_layer(w, device=DEV, sharp=True)
    layout = B.make_layout(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
    cap = B.cache_capacity(w.n_frames, w.tokens_per_frame, w.group_frames, w.retention)
    ws = B.make_workspace(layout, w.group_tokens, w.n_window)
    cache = B.Cache(layout, cap)
    out = torch.empty_like(q)

    def run():
        cache.reset()
        B.prefill_video(layout, w.n_frames, w.tokens_per_frame, w.group_frames, w.retention, "window_attn", q, k, v,
                        qw, cache, out, ws)

    run()                                                     # eager: also creates the library's streams
    torch.cuda.synchronize()
    want = (out.clone(), cache.k.clone(), cache.v.clone(), cache.pos.clone())
    final_len = cache.len
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    assert cache.len == final_len                             # the host-side length advanced during capture
    for replay in range(3):
        out.fill_(float("nan"))
        cache.k.zero_()
        cache.v.zero_()
        cache.pos.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (out, cache.k, cache.v, cache.pos)
        for a, b in zip(want, got):
            assert torch.equal(a, b), f"replay {replay}"
        run()                                                 # eager work between the replays
        torch.cuda.synchronize()
        for a, b in zip(want, got):
            assert torch.equal(a, b), f"eager after replay {replay}"


def test_capacity_and_unsupported_errors_leave_the_cache_alone():
    layout = B.make_layout(8, 2, 128, "bf16")
    n_g, keep = 256, 100
    k = torch.randn(n_g, 2, 128, device=DEV).bfloat16()
    v = torch.randn(n_g, 2, 128, device=DEV).bfloat16()
    s = torch.randn(2, n_g, device=DEV)
    cache = B.Cache(layout, 150)
    kept = torch.empty(2, keep, dtype=torch.int32, device=DEV)
    B.topk_compact(layout, s, k, v, keep, 0, cache, kept)
    assert cache.len == 100
    before = (cache.k.clone(), cache.pos.clone())
    with pytest.raises(B.QPError) as e:
        B.topk_compact(layout, s, k, v, keep, n_g, cache, kept)          # 100 + 100 > 150
    assert e.value.status == B.QP_ERR_CAPACITY and cache.len == 100
    torch.cuda.synchronize()
    assert torch.equal(cache.k, before[0]) and torch.equal(cache.pos, before[1])
    # neither a kept-index buffer nor a workspace is needed: selection and copy are one launch
    B.topk_compact(layout, s, k, v, 20, n_g, cache, None, None)
    torch.cuda.synchronize()
    assert cache.len == 120
    want = O.topk_select(s.double().cpu().numpy(), 20)
    np.testing.assert_array_equal(cache.pos.cpu().numpy()[:, 100:120], n_g + want)
    for h in range(2):
        assert torch.equal(cache.k[h, 100:120], k[torch.from_numpy(want[h]).to(DEV), h])
        assert torch.equal(cache.k[h, :100], before[0][h, :100])
    # forcing the MFMA kernel on a layout it does not take is refused, the scalar kernel takes it
    l64 = B.make_layout(4, 2, 64, "bf16")
    q64 = torch.randn(16, 4, 64, device=DEV).bfloat16()
    k64 = torch.randn(16, 2, 64, device=DEV).bfloat16()
    o64 = torch.empty_like(q64)
    B.select_attend_kernel(B.QP_ATTEND_MFMA)
    with pytest.raises(B.QPError) as e:
        B.group_attend(l64, q64, k64, k64, None, o64)
    assert e.value.status == B.QP_ERR_UNSUPPORTED
    B.select_attend_kernel(B.QP_ATTEND_AUTO)
    B.group_attend(l64, q64, k64, k64, None, o64)
    torch.cuda.synchronize()
    assert torch.isfinite(o64.float()).all()


def test_group_attend_largest_group():
    """The largest group the boundary accepts (32768 tokens), few heads: sampled rows against the oracle."""
    n_g, h_q, h_kv, d, c = B.QP_MAX_GROUP_TOKENS, 2, 1, 128, 100
    g = torch.Generator(device=DEV).manual_seed(3)
    mk = lambda *s: torch.randn(*s, generator=g, device=DEV).bfloat16()
    q, k, v = mk(n_g, h_q, d), mk(n_g, h_kv, d), mk(n_g, h_kv, d)
    layout = B.make_layout(h_q, h_kv, d, "bf16")
    cache = B.Cache(layout, c)
    cache.k.copy_(mk(h_kv, c, d))
    cache.v.copy_(mk(h_kv, c, d))
    cache.c.len = c
    out = torch.full_like(q, float("nan"))
    B.group_attend(layout, q, k, v, cache, out)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    rows = sample_rows(n_g, 20, np.random.default_rng(1))
    want = O.attend_group(_f64(q), _f64(k), _f64(v), _f64(cache.k), _f64(cache.v), rows=rows)
    assert_attn_close(_f64(out[rows]), want, "bf16", "largest group")


def test_prefill_video_failure_mid_loop_joins_streams_and_restores_the_cache_length():
    """A launch check that fails in the third group (forced from the host; every kernel still runs normally): the call
    reports QP_ERR_HIP, hands the cache back at its length at entry, and has joined its streams, so that the very next
    call on the same stream reproduces an undisturbed run bit for bit."""
    w = scaled(CONFIGS["cfg2_7b_32k"], n_frames=24, tokens_per_frame=64, group_frames=4)
    q, k, v, qw = make_layer(w, device=DEV, sharp=True)
    layout = B.make_layout(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
    cap = B.cache_capacity(w.n_frames, w.tokens_per_frame, w.group_frames, w.retention)
    ws = B.make_workspace(layout, w.group_tokens, w.n_window)
    cache = B.Cache(layout, cap)
    out = torch.empty_like(q)

    def run():
        cache.reset()
        B.prefill_video(layout, w.n_frames, w.tokens_per_frame, w.group_frames, w.retention, "window_attn", q, k, v,
                        qw, cache, out, ws)

    run()
    torch.cuda.synchronize()
    want = (out.clone(), cache.k.clone(), cache.v.clone(), cache.pos.clone())
    final_len = cache.len
    for nth in (1, 5, 8, 9):                                  # group 0's attention; group 1's scores; group 2's scores, top-k
        cache.reset()
        assert B.lib().qp_debug_fail_after(nth) == B.QP_OK
        try:
            with pytest.raises(B.QPError) as e:
                B.prefill_video(layout, w.n_frames, w.tokens_per_frame, w.group_frames, w.retention, "window_attn", q,
                                k, v, qw, cache, out, ws)
        finally:
            B.lib().qp_debug_fail_after(0)
        assert e.value.status == B.QP_ERR_HIP
        assert cache.len == 0                                 # restored, although earlier groups were appended
        run()                                                 # no synchronisation in between: ordered by the join
        torch.cuda.synchronize()
        assert cache.len == final_len
        for a, b in zip(want, (out, cache.k, cache.v, cache.pos)):
            assert torch.equal(a, b), f"after a failure at check {nth}"
