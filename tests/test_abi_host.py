"""Host-side checks of the C-ABI library that need no GPU: exports, host arithmetic, argument errors."""
import ctypes
import os
import re

import numpy as np
import pytest

from conftest import ROOT, read_golden
from oracle import qp_oracle as O
from paper_2505_16175_amd import binding as B
from paper_2505_16175_amd.workload import CONFIGS


def test_library_exports_every_declared_symbol():
    declared = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        header = open(os.path.join(ROOT, "include", name)).read()
        body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared |= set(re.findall(r"\b(qp_[a-z_0-9]+)\s*\((?!\*)", body))   # not the return type of a function-pointer typedef
    assert {"qp_group_attend", "qp_score_kv", "qp_topk_compact", "qp_prefill_video", "qp_layer_group"} <= declared
    handle = ctypes.CDLL(B.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(handle, name), f"{name} declared in include/ but not exported"
    assert declared == set(B.SIGNATURES), "binding and headers disagree on the entry points"
    assert B.version().startswith("quickprefill")


def test_group_bounds_match_the_oracle_and_a_hand_case():
    # hour-long config: 56 groups of 64 frames and one of 16 (3600 = 56 * 64 + 16)
    w = CONFIGS["cfg5_7b_hour_stack"]
    b = B.group_bounds(w.n_frames, w.tokens_per_frame, w.group_frames)
    assert len(b) == 57 and b[0] == (0, 8192) and b[-1] == (56 * 8192, 2048) and sum(n for _, n in b) == w.n_tokens
    for f, t, g in ((1, 1, 1), (7, 6, 3), (8, 16, 2), (5, 3, 9), (256, 128, 16), (3600, 128, 64)):
        assert B.group_bounds(f, t, g) == [tuple(x) for x in O.group_bounds(f, t, g)]
    lib = B.lib()
    assert lib.qp_group_bounds(0, 1, 1, None, None, 0) == -1
    assert lib.qp_group_bounds(4, 0, 1, None, None, 0) == -1
    assert lib.qp_group_bounds(4, 4, 0, None, None, 0) == -1
    assert lib.qp_group_bounds(1 << 20, 1 << 12, 1, None, None, 0) == -1      # token indices beyond int32
    first = (ctypes.c_int32 * 2)(-7, -7)                                       # fewer slots than groups: only those are written
    assert lib.qp_group_bounds(7, 6, 3, first, None, 1) == 3 and list(first) == [0, -7]


@pytest.mark.skipif(__import__("torch").cuda.is_available(), reason="needs a machine WITHOUT a GPU: there every launch fails")
def test_prefill_video_reports_a_failed_launch_and_leaves_the_cache_length():
    # Host code never dereferences the data pointers, so made-up aligned addresses do; without a device the first
    # launch fails, the call must say so and hand the cache back as it got it.
    L = B.make_layout(4, 2, 64, "f32")
    fake = 1 << 20
    c = B.qp_cache(fake, fake, fake, B.cache_capacity(8, 16, 2, 0.5) + 5, 5)
    st = B.lib().qp_prefill_video(ctypes.byref(L), 8, 16, 2, 0.5, 0, fake, fake, fake, None, 0, ctypes.byref(c), fake,
                                  fake, B.workspace_bytes(L, 32, 0), None)
    assert st == B.QP_ERR_HIP and c.len == 5 and B.last_hip_error() != 0


def test_debug_fail_after_arguments():
    assert B.lib().qp_debug_fail_after(-1) == B.QP_ERR_INVALID_ARG
    assert B.lib().qp_debug_fail_after(0) == B.QP_OK


def test_linear_plan_chunks_cover_the_contraction():
    """Host arithmetic of the projection launch: k chunks are non-empty and cover all 64-wide k-steps, the partial
    sums fit the scratch offered, launches that fill the GPU are never split, and without scratch nothing is."""
    offered = 32 << 20
    for m in (1, 7, 64, 128, 129, 300, 2048, 8192):
        for n, k in ((3584, 3584), (4608, 3584), (3584, 18944), (512, 1024), (8, 64), (8192, 29568), (264, 640)):
            p = B.linear_plan(m, n, k, offered)
            rows, steps = p["token_rows_per_tile"], k // 64
            if m <= 2:      # the weight-streaming kernel: 4 weight rows per workgroup, never split
                assert (rows, p["workgroups"], p["k_chunks"], p["scratch_bytes"]) == (m, n // 4, 1, 0)
                B.select_linear_tile(256)       # a pinned tiling keeps the call on the tiled kernel
                try:
                    p = B.linear_plan(m, n, k, offered)
                finally:
                    B.select_linear_tile(0)
                rows = p["token_rows_per_tile"]
            assert rows in (128, 256)
            tiles = -(-m // rows) * -(-n // 256)
            assert p["workgroups"] >= tiles and p["workgroups"] % 8 == 0
            c, per = p["k_chunks"], p["k_steps_per_chunk"]
            assert c >= 1 and (c - 1) * per < steps <= c * per
            if c > 1:
                assert tiles * 4 <= 256 and per >= 4 and c * tiles <= 256 + tiles
                assert p["scratch_bytes"] == c * m * n * 4 <= offered
            else:
                assert p["scratch_bytes"] == 0
            if tiles * 4 > 256:
                assert c == 1
            assert B.linear_plan(m, n, k, 0)["k_chunks"] == 1
    # the layer's text-chunk-shaped calls do split (single tokens stream the weights instead, see above)
    assert B.linear_plan(64, 3584, 18944, offered)["k_chunks"] >= 8
    assert B.linear_plan(7, 4608, 3584, offered)["k_chunks"] >= 8
    with pytest.raises(B.QPError):
        B.linear_plan(4, 8, 72)                                   # k not a multiple of 64


def test_layer_workspace_and_shape_errors():
    L = B.make_layout(28, 4, 128, "bf16")
    S = B.make_layer_shape(3584, 18944)
    n = B.layer_workspace_bytes(L, S, 2048, 64)
    acts = 2048 * 2 * (2 * 3584 + 2 * 28 * 128 + 2 * 4 * 128 + 18944)          # h (reused for h2), x1, q, attn, k, v, act
    split = 32 << 20                                                             # scratch of split contractions
    assert n >= acts + split + B.workspace_bytes(L, 2048, 64)
    assert n < acts + split + B.workspace_bytes(L, 2048, 64) + (4 << 20)
    # Appendix D.1 prices a group's activations at Q, K, V (query head count) + one score block per head for the
    # attention block and (2 d_model + 4 d_ff) per token for the MLP block; what the layer call keeps is below that
    # (one d_ff-wide tensor instead of four, K and V at the KV head count), and 1/G of the whole video's
    model_group = O.attn_activation_bytes(1, 2048, 28, 128, 1024, 1024) + O.mlp_activation_bytes(1, 2048, 3584, 18944)
    model_video = O.attn_activation_bytes(1, 32768, 28, 128, 1024, 1024) + O.mlp_activation_bytes(1, 32768, 3584, 18944)
    assert acts < model_group < model_video / 10
    assert B.layer_workspace_bytes(L, S, 0, 0) == 0
    assert B.layer_workspace_bytes(B.make_layout(28, 4, 64, "bf16"), S, 128, 0) == 0       # head_dim 128 only
    assert B.layer_workspace_bytes(L, B.make_layer_shape(3584, 18944, mrope_section=(16, 24, 20)), 128, 0) == 0
    assert B.layer_workspace_bytes(L, B.make_layer_shape(3584 + 8, 18944), 128, 0) == 0


def test_host_arithmetic_matches_oracle_and_golden():
    for n in (1, 2, 31, 100, 2048, 4096, 8192):
        for rho in (0.07, 0.1, 0.2, 0.25, 0.3, 0.5, 0.9, 1.0):
            assert B.keep_count(n, rho) == O.keep_count(n, rho)
    assert B.keep_count(0, 0.5) == 0 and B.keep_count(10, 0.0) == -1 and B.keep_count(10, 1.5) == -1
    for name, _, _, _, total in read_golden("cache_lengths.txt"):
        w = CONFIGS[name]
        assert B.cache_capacity(w.n_frames, w.tokens_per_frame, w.group_frames, w.retention) == int(total)
    assert B.cache_capacity(0, 1, 1, 0.5) == -1


def test_attend_plan_splits_only_the_last_round_of_a_long_launch():
    """Launches of more workgroups than compute units: when the last round of workgroups would fill only part of a KV
    head's compute units, exactly that round's row blocks are split, into as many chunks as make them fill the units
    evenly; full rounds, short caches and calls without scratch are left alone."""
    offered = 128 << 20
    L7 = B.make_layout(28, 4, 128, "bf16")                                  # 64 compute units per KV head
    p = B.attend_plan(L7, 8192, 24000, offered)                             # 224 row blocks per head: 3.5 rounds
    assert (p["split_row_blocks"], p["key_chunks"], p["mirrored_rows"]) == (32, 2, 0)
    assert p["workgroups"] == (192 + 32 * 2) * 4 and p["scratch_bytes"] == 2 * 4 * 8192 * 129 * 4
    assert p["tiles_per_chunk"] * 2 >= 375 > p["tiles_per_chunk"]
    p = B.attend_plan(L7, 4096, 24000, offered)                             # 112 per head: 1.75 rounds
    assert (p["split_row_blocks"], p["key_chunks"]) == (48, 4) and p["workgroups"] == (64 + 48 * 4) * 4
    assert p["scratch_bytes"] == 4 * 4 * 48 * 256 * 129 * 4
    assert B.attend_plan(L7, 8192, 24000, 32 << 20)["key_chunks"] == 1      # scratch too small for the partials
    assert B.attend_plan(L7, 8192, 24000, 0)["key_chunks"] == 1
    assert B.attend_plan(L7, 8192, 700, offered)["key_chunks"] == 1         # chunks would be shorter than 16 tiles
    assert B.attend_plan(L7, 9362, 24000, offered)["key_chunks"] == 1       # 256 per head: four full rounds
    L72 = B.make_layout(64, 8, 128, "bf16")                                 # 32 compute units per KV head
    assert B.attend_plan(L72, 4096, 16384, offered)["key_chunks"] == 1      # 128 per head: four full rounds
    assert B.attend_plan(L72, 3000, 16384, offered)["key_chunks"] == 1      # 94 per head: the last round is 30 / 32 full
    p = B.attend_plan(L72, 1100, 2100, offered)                             # 35 per head: 3 row blocks over 32 units
    assert p["split_row_blocks"] == 3 and p["key_chunks"] == 2
    for n_g in (2300, 2350, 3000, 4096, 5000, 8192, 20000, 32768):
        for c in (0, 1000, 1024, 2047, 2048, 5000, 9840, 46125, 200000):
            for L, r, h_kv, pool in ((L7, 7, 4, 64), (L72, 8, 8, 32)):
                p = B.attend_plan(L, n_g, c, offered)
                n_rb = -(-n_g * r // 256)
                s, per, rb = p["key_chunks"], p["tiles_per_chunk"], p["split_row_blocks"]
                if n_rb * h_kv <= 256 or s == 1:
                    assert s == 1 or rb == n_rb or p["mirrored_rows"] == 1
                    continue
                n_ct = -(-c // 64)
                assert 2 <= s <= 8 and rb == n_rb % pool and per >= 16
                assert (s - 1) * per < n_ct <= s * per                      # every chunk starts on an existing cache tile
                assert p["scratch_bytes"] == s * h_kv * min(n_g * r, rb * 256) * 129 * 4 <= offered
                assert -(-rb * s // pool) / s < 0.9                         # the split round is shorter than a whole one
                assert p["workgroups"] >= (n_rb - rb + rb * s) * h_kv


def test_attend_plan_invariants_on_random_shapes():
    """Whatever the shape: a split has at least two chunks, every chunk starts on an existing cache tile, the partials
    of the split rows fit the scratch that was offered, the grid holds every work item, and nothing is split without
    scratch."""
    rng = np.random.default_rng(20251128)
    for _ in range(3000):
        r = int(rng.choice([1, 2, 4, 7, 8, 16]))
        h_kv = int(rng.choice([1, 2, 3, 4, 8, 16]))
        n_g = int(rng.choice([1, 3, 33, 64, 100, 512, 1000, 2048, 2350, 4096, 8192, 20000, 32768]))
        c = int(rng.choice([0, 1, 63, 64, 65, 500, 1023, 1024, 5000, 24000, 46125, 150000]))
        offered = int(rng.choice([0, 1 << 20, 8 << 20, 32 << 20, 128 << 20]))
        L = B.make_layout(r * h_kv, h_kv, 128, "bf16")
        p = B.attend_plan(L, n_g, c, offered)
        rows = n_g * r
        if p["kernel"] == B.QP_ATTEND_MFMA_DECODE:
            assert rows <= 32
            continue
        assert p["kernel"] == B.QP_ATTEND_MFMA
        n_rb, n_ct = -(-rows // 256), -(-c // 64)
        s_, per, rb = p["key_chunks"], p["tiles_per_chunk"], p["split_row_blocks"]
        if s_ == 1:
            assert (per, rb, p["scratch_bytes"]) == (0, 0, 0)
        else:
            assert offered > 0 and 2 <= s_ <= 128 and 1 <= rb <= n_rb
            assert (s_ - 1) * per < n_ct <= s_ * per
            assert p["scratch_bytes"] == s_ * h_kv * min(rows, rb * 256) * 129 * 4 <= offered
            assert rb == n_rb or p["mirrored_rows"] == 0          # a partial split only with consecutive row blocks
        assert p["workgroups"] >= (n_rb - rb + rb * s_) * h_kv
        assert p["mirrored_rows"] == (1 if n_rb * h_kv <= 256 else 0)


def test_attend_plan_chunks_cover_the_cache_exactly():
    """Host arithmetic of the attention launch: when the cache is split over key chunks, every chunk is non-empty,
    the chunks tile the cache's 64-key tiles exactly, the scratch fits what was offered, and big launches never split."""
    L = B.make_layout(28, 4, 128, "bf16")
    offered = 32 << 20
    for n_g in (1, 2, 7, 64, 100, 128, 500, 2048, 8192):
        for c in (0, 1, 63, 64, 200, 256, 257, 1031, 5000, 9840, 46125, 200000):
            p = B.attend_plan(L, n_g, c, offered)
            rows_per_head = n_g * 7
            if rows_per_head <= 32:
                # decode-shaped: blocks of 32 keys (+ one block for the group's own keys) dealt to workgroups of 4
                # wavefronts; every workgroup gets at least one block, every wavefront of a full one too
                assert p["kernel"] == B.QP_ATTEND_MFMA_DECODE
                nb = (c + 31) // 32 + 1
                s, per = p["key_chunks"], p["tiles_per_chunk"]
                assert per >= 4 and (s - 1) * per < nb <= s * per and s == p["workgroups"]
                assert s * 4 <= 256 + 4                              # about one workgroup per compute unit at most
                assert p["scratch_bytes"] == (s * 4 * rows_per_head * 129 * 4 if s > 1 else 0) <= offered
                assert B.attend_plan(L, n_g, c, 0)["key_chunks"] == 1
                continue
            assert p["kernel"] == B.QP_ATTEND_MFMA
            real_wgs = ((rows_per_head + 127) // 128 + 1) // 2 * 4
            assert p["workgroups"] >= real_wgs and p["workgroups"] % 8 == 0
            n_ct = (c + 63) // 64
            s, per = p["key_chunks"], p["tiles_per_chunk"]
            if s == 1:
                assert per == 0 and p["scratch_bytes"] == 0
                # a small launch against a long cache must have split (enough scratch was offered for two chunks)
                if real_wgs < 128 and n_ct >= 4 and 2 * 4 * rows_per_head * 129 * 4 <= offered:
                    raise AssertionError(f"no split for n_g={n_g} c={c}")
            else:
                assert real_wgs < 128 and 2 <= s <= 128 and per >= 2
                assert (s - 1) * per < n_ct <= s * per          # every chunk starts on an existing cache tile
                assert p["scratch_bytes"] == s * 4 * rows_per_head * 129 * 4 <= offered
                assert real_wgs * s <= 2 * 256 + real_wgs       # about one workgroup per compute unit
            assert B.attend_plan(L, n_g, c, 0)["key_chunks"] == 1   # no scratch, no split
    assert B.attend_plan(L, 2048, 9840, offered)["mirrored_rows"] == 1      # 224 workgroups: one per CU, balanced
    assert B.attend_plan(L, 8192, 24000, offered)["mirrored_rows"] == 0     # 896 workgroups: longest first
    assert B.attend_plan(B.make_layout(4, 2, 64, "f32"), 32, 64, offered)["kernel"] == B.QP_ATTEND_SCALAR
    with pytest.raises(B.QPError):
        B.attend_plan(L, 0, 10, 0)
    with pytest.raises(B.QPError):
        B.attend_plan(L, 16, -1, 0)


def test_argument_errors_are_caught_on_the_host():
    lib = B.lib()
    L = B.make_layout(28, 4, 128, "bf16")
    fake = ctypes.c_void_p(4096)            # aligned, never dereferenced: every case fails validation first
    cache = B.qp_cache(4096, 8192, 12288, 100, 0)
    ref, refc = ctypes.byref(L), ctypes.byref(cache)
    ws = ctypes.c_void_p(1 << 20)
    # NULL / misaligned / bad sizes
    assert lib.qp_group_attend(ref, None, fake, fake, 16, None, fake, None, None, 0, None) == B.QP_ERR_INVALID_ARG
    assert lib.qp_group_attend(ref, ctypes.c_void_p(4098), fake, fake, 16, None, fake, None, None, 0, None) == B.QP_ERR_INVALID_ARG
    assert lib.qp_group_attend(ref, fake, fake, fake, 0, None, fake, None, None, 0, None) == B.QP_ERR_INVALID_ARG
    assert lib.qp_group_attend(ref, fake, fake, fake, B.QP_MAX_GROUP_TOKENS + 1, None, fake, None, None, 0, None) == B.QP_ERR_UNSUPPORTED
    bad = B.make_layout(28, 5, 128, "bf16")
    assert lib.qp_group_attend(ctypes.byref(bad), fake, fake, fake, 16, None, fake, None, None, 0, None) == B.QP_ERR_INVALID_ARG
    odd = B.make_layout(28, 4, 96, "bf16")
    assert lib.qp_group_attend(ctypes.byref(odd), fake, fake, fake, 16, None, fake, None, None, 0, None) == B.QP_ERR_UNSUPPORTED
    # scoring: window rule without a window, unknown rule, small workspace
    assert lib.qp_score_kv(ref, B.QP_SCORE_WINDOW_ATTN, fake, fake, 16, None, 0, fake, ws, 1 << 20, None) == B.QP_ERR_INVALID_ARG
    assert lib.qp_score_kv(ref, 7, fake, fake, 16, None, 0, fake, ws, 1 << 20, None) == B.QP_ERR_INVALID_ARG
    assert lib.qp_score_kv(ref, B.QP_SCORE_WINDOW_ATTN, fake, fake, 16, fake, 64, fake, ws, 16, None) == B.QP_ERR_CAPACITY
    assert lib.qp_score_kv(ref, B.QP_SCORE_KEY_NORM_SMALL, None, fake, 16, None, 0, fake, None, 0, None) == B.QP_ERR_INVALID_ARG
    # top-k: keep out of range, capacity overflow; the cache length must not move
    assert lib.qp_topk_compact(ref, fake, fake, fake, 16, 0, 0, refc, None, None, 0, None) == B.QP_ERR_INVALID_ARG
    assert lib.qp_topk_compact(ref, fake, fake, fake, 16, 17, 0, refc, None, None, 0, None) == B.QP_ERR_INVALID_ARG
    cache.len = 95
    assert lib.qp_topk_compact(ref, fake, fake, fake, 16, 6, 0, refc, None, None, 0, None) == B.QP_ERR_CAPACITY
    assert cache.len == 95
    cache.len = 0
    # whole-video call: bad retention, cache too small, workspace too small
    args = (fake, fake, fake, fake, 64, refc, fake)
    assert lib.qp_prefill_video(ref, 8, 16, 2, 0.0, 0, *args, ws, 1 << 20, None) == B.QP_ERR_INVALID_ARG
    assert lib.qp_prefill_video(ref, 8, 16, 2, 1.0, 0, *args, ws, 1 << 20, None) == B.QP_ERR_CAPACITY   # needs 128 > 100
    assert lib.qp_prefill_video(ref, 8, 16, 2, 0.5, 2, *args, ws, 64, None) == B.QP_ERR_CAPACITY
    assert lib.qp_prefill_video(ref, 8, 16, 2, 0.5, 2, fake, fake, fake, None, 0, refc, fake, ws, 1 << 20, None) == B.QP_ERR_INVALID_ARG
    assert cache.len == 0
    assert lib.qp_select_attend_kernel(9) == B.QP_ERR_INVALID_ARG
    assert B.workspace_bytes(L, 0, 0) == 0 and B.workspace_bytes(L, 8192, 64) > 4 * 8192 * 4
    for s in range(5):
        assert B.status_string(s)


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_16175_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("the CPU oracle's tests", ""), f


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: `bench.py --gpus N` with N > 1 says so and exits without touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_e4m3_conversions_match_the_oracle_for_every_input():
    """The library's bf16 -> E4M3 conversion (the routine its compaction kernel runs, here through its host entry
    point) against the oracle's rounding for all 65536 bf16 bit patterns, and the decode for all 256 codes."""
    import numpy as np
    import torch
    lib = B.lib()
    bits = np.arange(65536, dtype=np.uint32)
    with np.errstate(invalid="ignore"):                       # signalling-NaN patterns are among the inputs
        vals = (bits << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    codes = np.array([lib.qp_e4m3_from_bf16(int(b)) for b in bits], dtype=np.uint32)
    back = np.array([lib.qp_bf16_from_e4m3(int(c)) for c in range(256)], dtype=np.uint32)
    decoded = (back << 16).astype(np.uint32).view(np.float32).astype(np.float64)          # value of every code
    # decode: the format's definition, and the library format torch implements
    want_dec = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(np.isnan(decoded), np.isnan(want_dec))
    ok = ~np.isnan(want_dec)
    np.testing.assert_array_equal(decoded[ok], want_dec[ok])
    assert (np.signbit(decoded) == (np.arange(256) >= 128)).all()
    # encode: equals the oracle's rounding (nearest, ties to even, saturating), sign carried, NaN to the NaN code
    nan = np.isnan(vals)
    assert ((codes[nan] & 0x7f) == 0x7f).all()
    got = decoded[codes[~nan]]
    np.testing.assert_array_equal(got, O.fp8_e4m3_round(vals[~nan]))
    np.testing.assert_array_equal(np.signbit(got), np.signbit(vals[~nan]))
