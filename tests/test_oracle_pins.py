"""CPU pins of the fp64 oracle: each check ties an oracle function to something other than itself.

Brute force / library routines / closed forms / the paper's printed figures / hand-computed
examples / invariants, chosen so that a dropped term, a wrong sign or index, or a transposed
operand in the oracle fails at least one of them.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from conftest import read_golden
from oracle import qp_oracle as O

RNG = np.random.default_rng(7)


def _rand(*shape, sharp=3.0):
    return RNG.standard_normal(shape) * sharp


# ----------------------------------------------------------------------------- attention
def _brute_attend(q_g, k_g, v_g, ck, cv, scale):
    """Textbook attention: full masked logit matrix, library softmax, per scalar loops over heads."""
    n_g, h_q, d = q_g.shape
    h_kv = k_g.shape[1]
    r = h_q // h_kv
    c = ck.shape[1]
    out = np.zeros((n_g, h_q, d))
    for qh in range(h_q):
        h = qh // r
        for i in range(n_g):
            logits, vals = [], []
            for e in range(c):
                logits.append(scale * sum(q_g[i, qh, x] * ck[h, e, x] for x in range(d)))
                vals.append(cv[h, e])
            for j in range(i + 1):
                logits.append(scale * sum(q_g[i, qh, x] * k_g[j, h, x] for x in range(d)))
                vals.append(v_g[j, h])
            p = scipy.special.softmax(np.array(logits))
            out[i, qh] = sum(pj * vj for pj, vj in zip(p, vals))
    return out


@pytest.mark.parametrize("n_g,h_q,h_kv,d,c", [(5, 4, 2, 3, 0), (6, 6, 2, 4, 7), (1, 2, 1, 2, 3), (9, 3, 3, 5, 1)])
def test_attend_matches_brute_force(n_g, h_q, h_kv, d, c):
    q, k, v = _rand(n_g, h_q, d), _rand(n_g, h_kv, d), _rand(n_g, h_kv, d)
    ck, cv = _rand(h_kv, c, d), _rand(h_kv, c, d)
    scale = 0.37
    got, lse = O.attend_group(q, k, v, ck, cv, scale, return_lse=True)
    want = _brute_attend(q, k, v, ck, cv, scale)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    # lse against scipy's logsumexp on one row
    qh, i = h_q - 1, n_g - 1
    h = qh // (h_q // h_kv)
    keys = np.concatenate([ck[h], k[: i + 1, h]])
    np.testing.assert_allclose(lse[qh, i], scipy.special.logsumexp(scale * keys @ q[i, qh]), atol=1e-12)


def _sdpa_causal(q, k, v, scale):
    """Full causal attention over all tokens by the library routine (fp64), GQA by head repetition."""
    n, h_q, d = q.shape
    r = h_q // k.shape[1]
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, r, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, r, axis=1)).permute(1, 0, 2)[None]
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


@pytest.mark.parametrize("group_frames", [1, 2, 3, 8])
@pytest.mark.parametrize("rule", O.RULES)
def test_retention_one_is_full_causal_prefill(group_frames, rule):
    f, t, h_q, h_kv, d = 8, 5, 4, 2, 8
    q, k, v, qw = _rand(f * t, h_q, d), _rand(f * t, h_kv, d), _rand(f * t, h_kv, d), _rand(3, h_q, d)
    scale = 1 / math.sqrt(d)
    out, ck, cv, pos, _ = O.prefill_video(q, k, v, qw, f, t, group_frames, 1.0, rule)
    np.testing.assert_allclose(out, _sdpa_causal(q, k, v, scale), atol=1e-12)
    # nothing pruned: cache is the whole K/V in order
    assert (pos == np.arange(f * t)[None, :]).all()
    np.testing.assert_array_equal(ck, k.transpose(1, 0, 2))
    np.testing.assert_array_equal(cv, v.transpose(1, 0, 2))


@pytest.mark.parametrize("rho", [0.1, 0.5, 0.9])
def test_single_group_is_full_causal_for_any_retention(rho):
    f, t, h_q, h_kv, d = 4, 6, 6, 3, 4
    q, k, v = _rand(f * t, h_q, d), _rand(f * t, h_kv, d), _rand(f * t, h_kv, d)
    out, *_ = O.prefill_video(q, k, v, None, f, t, f, rho, "key_norm_small")
    np.testing.assert_allclose(out, _sdpa_causal(q, k, v, 1 / math.sqrt(d)), atol=1e-12)


def test_attend_invariants():
    n_g, h_q, h_kv, d, c = 12, 4, 2, 6, 9
    q, k, v = _rand(n_g, h_q, d), _rand(n_g, h_kv, d), _rand(n_g, h_kv, d)
    ck, cv = _rand(h_kv, c, d), _rand(h_kv, c, d)
    base = O.attend_group(q, k, v, ck, cv)
    # first token with an empty cache returns its own value vector
    first = O.attend_group(q, k, v, None, None)
    r = h_q // h_kv
    for qh in range(h_q):
        np.testing.assert_allclose(first[0, qh], v[0, qh // r], atol=1e-15)
    # convex combination: inside the per-coordinate hull of the visible values
    for qh in range(h_q):
        h = qh // r
        for i in range(n_g):
            vis = np.concatenate([cv[h], v[: i + 1, h]])
            assert (base[i, qh] <= vis.max(0) + 1e-12).all() and (base[i, qh] >= vis.min(0) - 1e-12).all()
    # permuting the cache entries (keys and values together) changes nothing
    perm = RNG.permutation(c)
    np.testing.assert_allclose(O.attend_group(q, k, v, ck[:, perm], cv[:, perm]), base, atol=1e-12)
    # a future token has no influence (causality): change the last group token
    k2, v2 = k.copy(), v.copy()
    k2[-1] += 5.0
    v2[-1] -= 3.0
    np.testing.assert_array_equal(O.attend_group(q, k2, v2, ck, cv)[:-1], base[:-1])
    # the cache IS visible to every row: removing it changes row 0
    assert np.abs(O.attend_group(q, k, v, None, None)[0] - base[0]).max() > 1e-3
    # swapping K and V operands is detected: the result changes
    assert np.abs(O.attend_group(q, v, k, cv, ck) - base).max() > 1e-3
    # rows= evaluates exactly those rows
    rows = [0, 5, 11]
    np.testing.assert_array_equal(O.attend_group(q, k, v, ck, cv, rows=rows), base[rows])
    # default scale is 1/sqrt(d)
    np.testing.assert_array_equal(O.attend_group(q, k, v, ck, cv, scale=1 / math.sqrt(d)), base)
    # GQA mapping: query head qh uses KV head qh // R -> equal to MHA with repeated KV heads
    mha = O.attend_group(q, np.repeat(k, r, 1), np.repeat(v, r, 1), np.repeat(ck, r, 0), np.repeat(cv, r, 0))
    np.testing.assert_allclose(mha, base, atol=1e-13)


def test_attention_over_key_chunks_merges_by_log_sum_exp():
    """The identity behind a key split: softmax attention over a key set equals the merge of the attentions over a
    partition of it, weighted by exp(lse_chunk - lse). Pins the oracle's lse output and is what the kernel's
    split-and-merge path relies on (each chunk starts on cache entries; the last takes the group's own keys)."""
    n_g, h_q, h_kv, d, c = 5, 6, 2, 8, 23
    q, k, v = _rand(n_g, h_q, d), _rand(n_g, h_kv, d), _rand(n_g, h_kv, d)
    ck, cv = _rand(h_kv, c, d), _rand(h_kv, c, d)
    whole, lse = O.attend_group(q, k, v, ck, cv, return_lse=True)
    # lse against its definition on one row: head 3 (KV head 1), token 2 sees the cache and group tokens 0..2
    logits = np.concatenate([ck[1] @ q[2, 3], k[:3, 1] @ q[2, 3]]) / math.sqrt(d)
    assert abs(lse[3, 2] - math.log(np.exp(logits).sum())) < 1e-12
    # chunks: cache [0,7), cache [7,16), cache [16,23) + the group itself. A cache-only chunk has no causal part; the
    # oracle always adds the group's own keys, so each row is run as a one-token group whose own key and value are
    # zero (logit 0, value 0) and that dummy key's share is then removed exactly
    cuts = [(0, 7), (7, 16), (16, 23)]
    parts = []
    for i, (a, b) in enumerate(cuts):
        if i < len(cuts) - 1:
            o = np.zeros((n_g, h_q, d))
            l = np.zeros((h_q, n_g))
            zero = np.zeros((1, h_kv, d))
            for t in range(n_g):
                oo, ll = O.attend_group(q[t:t + 1], zero, zero, ck[:, a:b], cv[:, a:b], return_lse=True)
                # remove the dummy key's contribution exactly: its logit is 0, its value 0
                w_dummy = np.exp(0.0 - ll[:, 0])                       # weight the dummy key received
                o[t] = oo[0] / (1.0 - w_dummy)[:, None]
                l[:, t] = ll[:, 0] + np.log1p(-w_dummy)
            parts.append((o, l))
        else:
            parts.append(O.attend_group(q, k, v, ck[:, a:b], cv[:, a:b], return_lse=True))
    lse_all = np.logaddexp.reduce(np.stack([l for _, l in parts]), axis=0)
    merged = sum(o * np.exp(l - lse_all).T[:, :, None] for o, l in parts)
    np.testing.assert_allclose(lse_all, lse, atol=1e-12)
    np.testing.assert_allclose(merged, whole, atol=1e-12)


def test_hand_example_whole_path():
    rows = {r[0]: r[1].split() for r in read_golden("hand_example_path.txt")}
    k = np.log(np.array([float(x) for x in rows["k_exp"]])).reshape(4, 1, 1)
    v = np.array([float(x) for x in rows["v"]]).reshape(4, 1, 1)
    q = np.ones((4, 1, 1))
    for rule, pre in (("key_norm_small", ""), ("value_norm", "vn_")):
        out, ck, cv, pos, sel = O.prefill_video(q, k, v, None, 4, 1, 2, 0.5, rule, scale=1.0)
        want = [Fraction(int(a), int(b)) for a, b in zip(rows[pre + "out_num"], rows[pre + "out_den"])]
        np.testing.assert_allclose(out[:, 0, 0], [float(x) for x in want], atol=1e-14)
        assert pos[0].tolist() == [int(x) for x in rows[pre + "kept_pos"]]
        np.testing.assert_array_equal(ck[0, :, 0], k[pos[0], 0, 0])
        np.testing.assert_array_equal(cv[0, :, 0], v[pos[0], 0, 0])


# ----------------------------------------------------------------------------- scores
def test_norm_scores_closed_form():
    k = np.zeros((3, 2, 4))
    k[0, 0] = [3, 4, 0, 0]          # 5
    k[1, 0] = [1, 2, 2, 0]          # 3
    k[2, 0] = [0, 0, 0, -7]         # 7
    k[0, 1] = [2, 3, 6, 0]          # 7
    k[1, 1] = [1, 1, 1, 1]          # 2
    k[2, 1] = [0, 0, 0, 0]          # 0
    want = np.array([[5, 3, 7], [7, 2, 0]], dtype=float)
    np.testing.assert_allclose(O.score_kv("key_norm_small", k, None), -want, atol=1e-15)
    np.testing.assert_allclose(O.score_kv("value_norm", k, k), want, atol=1e-15)
    # the key rule reads K and the value rule reads V, not the other way round
    v = 2 * k
    np.testing.assert_allclose(O.score_kv("value_norm", k, v), 2 * want, atol=1e-15)
    np.testing.assert_allclose(O.score_kv("key_norm_small", k, v), -want, atol=1e-15)
    # library cross-check
    x = _rand(17, 3, 9)
    np.testing.assert_allclose(O.score_kv("value_norm", x, x), np.linalg.norm(x, axis=2).T, atol=1e-13)


def test_norm_rules_are_complements():
    x = _rand(40, 2, 8)
    for k in (1, 7, 20, 39):
        small = O.topk_select(O.score_kv("key_norm_small", x, x), 40 - k)
        large = O.topk_select(O.score_kv("value_norm", x, x), k)
        for h in range(2):
            assert sorted(set(small[h]) | set(large[h])) == list(range(40))
            assert not (set(small[h]) & set(large[h]))


def test_window_score_brute_force_and_mass():
    n_g, h_q, h_kv, d, w = 11, 6, 2, 5, 4
    k, qw = _rand(n_g, h_kv, d, sharp=1.0), _rand(w, h_q, d, sharp=1.0)
    scale = 0.6
    s = O.score_kv("window_attn", k, None, qw, scale)
    r = h_q // h_kv
    want = np.zeros((h_kv, n_g))
    for qh in range(h_q):
        for t in range(w):
            logits = np.array([scale * float(np.dot(qw[t, qh], k[j, qh // r])) for j in range(n_g)])
            want[qh // r] += scipy.special.softmax(logits)
    np.testing.assert_allclose(s, want, atol=1e-13)
    # every softmax row has mass 1: total mass per KV head is R * W
    np.testing.assert_allclose(s.sum(axis=1), r * w, atol=1e-12)
    # zero queries -> uniform mass -> all ties -> the first k tokens survive
    s0 = O.score_kv("window_attn", k, None, np.zeros_like(qw), scale)
    np.testing.assert_allclose(s0, r * w / n_g, atol=1e-15)
    assert (O.topk_select(s0, 4) == np.arange(4)[None]).all()
    # one query, one head: the ranking is that of the raw logits (softmax is monotone)
    k1, q1 = _rand(n_g, 1, d), _rand(1, 1, d)
    s1 = O.score_kv("window_attn", k1, None, q1)
    assert (np.argsort(-s1[0], kind="stable") == np.argsort(-(k1[:, 0] @ q1[0, 0]), kind="stable")).all()
    # default scale is 1/sqrt(d)
    np.testing.assert_array_equal(O.score_kv("window_attn", k, None, qw), O.score_kv("window_attn", k, None, qw, d ** -0.5))
    # the window score does not depend on V
    np.testing.assert_array_equal(O.score_kv("window_attn", k, _rand(n_g, h_kv, d), qw, scale), s)


# ----------------------------------------------------------------------------- top-k
def test_window_logit_rule_brute_force_and_properties():
    """The softmax-free variant of the attention-score rule: element-wise brute force, linearity in the window
    queries, and agreement of its ranking with the softmax rule's when there is one query row and one query head per
    KV head (softmax is monotone in the logit)."""
    n_g, h_q, h_kv, d, w = 9, 4, 2, 5, 3
    k, qw = _rand(n_g, h_kv, d), _rand(w, h_q, d)
    got = O.score_kv("window_logit", k, None, qw)
    r = h_q // h_kv
    for h in range(h_kv):
        for j in range(n_g):
            acc = 0.0
            for t in range(w):
                for qh in range(h * r, (h + 1) * r):
                    acc += sum(qw[t, qh, e] * k[j, h, e] for e in range(d)) / math.sqrt(d)
            assert abs(got[h, j] - acc) < 1e-12
    qw2 = _rand(w, h_q, d)
    np.testing.assert_allclose(O.score_kv("window_logit", k, None, qw + qw2),
                               got + O.score_kv("window_logit", k, None, qw2), atol=1e-12)
    np.testing.assert_allclose(O.score_kv("window_logit", k, None, qw, scale=0.5),
                               0.5 * math.sqrt(d) * got, atol=1e-12)
    one = _rand(1, h_kv, d)                                    # W = 1, R = 1
    a = O.score_kv("window_logit", k, None, one)
    b = O.score_kv("window_attn", k, None, one)
    for h in range(h_kv):
        assert (np.argsort(-a[h], kind="stable") == np.argsort(-b[h], kind="stable")).all()
    for keep in (1, 4, n_g):
        np.testing.assert_array_equal(O.topk_select(a, keep), O.topk_select(b, keep))


def test_head_shared_selection():
    """One index set per group: every head's scores are replaced by the sum over heads, so the per-head TopK agrees
    across heads and equals the TopK of the summed scores; with one head nothing changes."""
    s = _rand(3, 11)
    shared = O.share_scores_across_heads(s)
    np.testing.assert_allclose(shared[0], s[0] + s[1] + s[2], atol=1e-15)
    assert (shared == shared[0]).all()
    sel = O.topk_select(shared, 4)
    assert (sel == sel[0]).all()
    np.testing.assert_array_equal(sel[0], O.topk_select((s[0] + s[1] + s[2])[None], 4)[0])
    np.testing.assert_array_equal(O.share_scores_across_heads(s[:1]), s[:1])
    # a token that one head loves and the others ignore is kept for all of them
    s2 = np.zeros((3, 6))
    s2[1, 4] = 10.0
    assert 4 in O.topk_select(O.share_scores_across_heads(s2), 1)[2]


def test_topk_hand_cases():
    for rule, vals, k, want in read_golden("topk_hand_cases.txt"):
        x = np.array([float(t) for t in vals.split()])
        if rule == "score":
            s = x[None, :]
        else:
            vec = x.reshape(-1, 1, 1)            # head_dim 1: the norm is |x|
            s = O.score_kv(rule, vec, vec)
        got = O.topk_select(s, int(k))[0].tolist()
        assert got == [int(t) for t in want.split()], (rule, vals, k)


def test_topk_equals_stable_sort_and_is_nested():
    for n in (5, 64, 65, 300):
        s = np.round(_rand(3, n), 1)             # coarse values -> many ties
        prev = [set() for _ in range(3)]
        for k in range(1, n + 1, max(1, n // 7)):
            got = O.topk_select(s, k)
            for h in range(3):
                want = np.sort(np.argsort(-s[h], kind="stable")[:k])
                assert (got[h] == want).all()
                assert (np.diff(got[h]) > 0).all()
                assert prev[h] <= set(got[h])
                prev[h] = set(got[h])


def test_keep_count_and_cache_lengths():
    assert O.keep_count(100, 0.07) == 7          # 0.07*100 = 7.000000000000001 must not round up
    assert O.keep_count(10, 0.25) == 3
    assert O.keep_count(10, 1.0) == 10
    assert O.keep_count(10, 1e-6) == 1
    assert O.keep_count(0, 0.5) == 0
    from paper_2505_16175_amd.workload import CONFIGS
    for name, n_g, k, g, total in read_golden("cache_lengths.txt"):
        w = CONFIGS[name]
        assert w.group_tokens == int(n_g)
        assert O.keep_count(int(n_g), w.retention) == int(k)
        bounds = O.group_bounds(w.n_frames, w.tokens_per_frame, w.group_frames)
        assert len(bounds) == int(g) == -(-w.n_frames // w.group_frames)
        assert sum(n for _, n in bounds) == w.n_tokens
        assert O.final_cache_len(w.n_frames, w.tokens_per_frame, w.group_frames, w.retention) == int(total)


def test_path_counts_positions_and_copy():
    f, t, g, rho = 7, 6, 3, 0.4                  # ragged last group: 1 frame
    h_q, h_kv, d = 4, 2, 4
    q, k, v, qw = _rand(f * t, h_q, d), _rand(f * t, h_kv, d), _rand(f * t, h_kv, d), _rand(5, h_q, d)
    for rule in O.RULES:
        out, ck, cv, pos, sel = O.prefill_video(q, k, v, qw, f, t, g, rho, rule)
        sizes = [18, 18, 6]
        assert [n for _, n, _, _ in sel] == sizes
        assert [i.shape[1] for _, _, i, _ in sel] == [math.ceil(rho * n - 1e-9) for n in sizes] == [8, 8, 3]
        assert pos.shape == (h_kv, 19)
        for h in range(h_kv):
            assert (np.diff(pos[h]) > 0).all()
            np.testing.assert_array_equal(ck[h], k[pos[h], h])
            np.testing.assert_array_equal(cv[h], v[pos[h], h])
        lo = 0
        for (base, n, idx, _) in sel:
            kk = idx.shape[1]
            assert ((pos[:, lo:lo + kk] >= base) & (pos[:, lo:lo + kk] < base + n)).all()
            lo += kk
        # select_all_groups / gather_cache reproduce the sequential path's cache
        sel2 = O.select_all_groups(k, v, qw, f, t, g, rho, rule)
        ck2, cv2, pos2 = O.gather_cache(k, v, sel2, len(sel2))
        np.testing.assert_array_equal(pos2, pos)
        np.testing.assert_array_equal(ck2, ck)
        np.testing.assert_array_equal(cv2, cv)
        # and the attention of a later group over that cache reproduces the path's output
        base, n, _, _ = sel[2]
        ck1, cv1, _ = O.gather_cache(k, v, sel2, 2)
        np.testing.assert_array_equal(O.attend_group(q[base:], k[base:], v[base:], ck1, cv1), out[base:])


def test_pruned_tokens_are_invisible_later():
    """A token dropped from the cache must not influence later groups; a kept one must."""
    f, t, g = 4, 4, 2
    q = _rand(16, 2, 4)
    k = _rand(16, 1, 4)
    v = _rand(16, 1, 4)
    out, _, _, pos, sel = O.prefill_video(q, k, v, None, f, t, g, 0.25, "value_norm")
    kept0 = set(sel[0][2][0].tolist())
    dropped = next(j for j in range(8) if j not in kept0)
    kept = next(iter(kept0))
    v2 = v.copy()
    v2[dropped] *= 0.5                           # smaller norm: stays dropped
    out2, *_ = O.prefill_video(q, k, v2, None, f, t, g, 0.25, "value_norm")
    np.testing.assert_array_equal(out2[8:], out[8:])
    v3 = v.copy()
    v3[kept] *= 1.5                              # larger norm: stays kept, values change downstream
    out3, *_ = O.prefill_video(q, k, v3, None, f, t, g, 0.25, "value_norm")
    assert np.abs(out3[8:] - out[8:]).max() > 1e-6


# ----------------------------------------------------------------------------- memory models
def test_memory_models_match_paper_figures():
    fn = {"attn_activation": O.attn_activation_bytes, "attn_activation_grouped": O.attn_activation_bytes,
          "mlp_activation": O.mlp_activation_bytes, "mlp_activation_grouped": O.mlp_activation_bytes,
          "kv_cache": O.kv_cache_bytes}
    for name, params, value, tol in read_golden("paper_memory_figures.txt"):
        kw = {p.split("=")[0]: int(p.split("=")[1]) for p in params.split()}
        gib = fn[name](**kw) / 2 ** 30
        assert abs(gib - float(value)) <= float(tol), (name, gib)
    # pruning shrinks the cache by 1/rho (Sec. 3.2)
    assert O.kv_cache_bytes(28, 1000, 8, 128, 2, retention=0.25) * 4 == O.kv_cache_bytes(28, 1000, 8, 128, 2)


# --------------------------------------------------------------------------- the 8-bit cache variant
def _e4m3_values():
    """Every finite value of the format, decoded from its bit patterns by the format's definition."""
    vals = []
    for code in range(128):
        e, m = code >> 3, code & 7
        if e == 15 and m == 7:
            continue                                           # NaN
        vals.append((m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7))
    return np.array(sorted(vals))


def test_fp8_rounding_hand_cases():
    for x, want, why in read_golden("fp8_e4m3_hand_cases.txt"):
        got = float(O.fp8_e4m3_round(float(x)))
        assert got == float(want), (x, got, want, why)
        assert float(O.fp8_e4m3_round(-float(x))) == -float(want)        # odd symmetry


def test_fp8_rounding_is_the_nearest_representable_value_ties_to_even():
    vals = _e4m3_values()
    assert len(vals) == 127 and vals[0] == 0.0 and vals[1] == 2.0 ** -9 and vals[-1] == 448.0
    rng = np.random.default_rng(8)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-4, 3, 4000), rng.uniform(-460, 460, 2000),
                        (vals[:-1] + vals[1:]) / 2, vals])     # random values, every halfway point, every value itself
    got = O.fp8_e4m3_round(x)
    assert np.isin(np.abs(got), vals).all()
    # brute force: nearest value by distance; at exact halfway points the one with the even code
    a = np.minimum(np.abs(x), 448.0)
    d = np.abs(a[:, None] - vals[None, :])
    best = d.min(axis=1)
    for i in range(len(x)):
        cand = np.flatnonzero(d[i] == best[i])
        pick = cand[0] if len(cand) == 1 else [c for c in cand if c % 2 == 0][0]   # index in the sorted table = code
        assert abs(got[i]) == vals[pick], (x[i], got[i], vals[pick])
    np.testing.assert_array_equal(O.fp8_e4m3_round(got), got)                       # idempotent
    xs = np.sort(x)
    assert (np.diff(O.fp8_e4m3_round(xs)) >= 0).all()                               # monotone
    assert np.isnan(O.fp8_e4m3_round(np.nan))


def test_fp8_rounding_matches_the_library_cast_inside_the_range():
    rng = np.random.default_rng(9)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-4, 3, 20000), rng.uniform(-448, 448, 5000)])
    x = x[np.abs(x) <= 448.0].astype(np.float32)                # the library cast does not saturate; inside the range they agree
    want = torch.tensor(x).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.fp8_e4m3_round(x.astype(np.float64)), want)


def test_fp8_cache_rounds_stored_rows_only():
    """With the 8-bit cache the kept sets, the first group's outputs and the group's own keys are untouched; the cache
    holds the rounded rows, and later groups attend to exactly those."""
    from paper_2505_16175_amd.workload import CONFIGS, make_layer, scaled, to_f64
    w = scaled(CONFIGS["cfg1_tiny_f32"], n_frames=6)
    q, k, v, qw = (to_f64(t) for t in make_layer(w, sharp=True))
    args = (w.n_frames, w.tokens_per_frame, w.group_frames, w.retention, "key_norm_small")
    out, ck, cv, pos, sel = O.prefill_video(q, k, v, qw, *args)
    out8, ck8, cv8, pos8, sel8 = O.prefill_video(q, k, v, qw, *args, cache_format="fp8_e4m3")
    np.testing.assert_array_equal(pos8, pos)
    np.testing.assert_array_equal(ck8, O.fp8_e4m3_round(ck))
    np.testing.assert_array_equal(cv8, O.fp8_e4m3_round(cv))
    n0 = w.group_tokens
    np.testing.assert_array_equal(out8[:n0], out[:n0])                        # the first group sees no cache
    assert np.abs(out8[n0:] - out[n0:]).max() > 1e-4                          # later groups see rounded rows
    # later groups attend to the rounded cache and their own exact K, V
    g1 = slice(n0, 2 * n0)
    gk, gv, _ = O.gather_cache(k, v, sel8, 1, cache_format="fp8_e4m3")
    np.testing.assert_array_equal(gk, ck8[:, :gk.shape[1]])
    np.testing.assert_allclose(out8[g1], O.attend_group(q[g1], k[g1], v[g1], gk, gv), atol=1e-15)
    # bytes: one per element instead of the inputs' (the bytes factor of the cache-memory equation of App. D.2)
    assert O.kv_cache_bytes(1, pos.shape[1], w.n_kv_heads, w.head_dim, 1) * 2 == O.kv_cache_bytes(1, pos.shape[1], w.n_kv_heads, w.head_dim, 2)
