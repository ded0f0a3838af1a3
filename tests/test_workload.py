"""The seeded input generator: shapes, reproducibility and the statistics the recipe promises."""
import math

import numpy as np
import torch

from paper_2505_16175_amd.workload import CONFIGS, make_layer, scaled, to_f64


def test_tiny_config_shapes_and_reproducibility():
    w = CONFIGS["cfg1_tiny_f32"]
    q, k, v, qw = make_layer(w)
    assert q.shape == (128, 4, 64) and k.shape == (128, 2, 64) and v.shape == (128, 2, 64) and qw.shape == (16, 4, 64)
    assert q.dtype == torch.float32
    q2, k2, v2, qw2 = make_layer(w)
    assert torch.equal(q, q2) and torch.equal(k, k2) and torch.equal(v, v2) and torch.equal(qw, qw2)
    q3, *_ = make_layer(w, layer=1)
    assert not torch.equal(q, q3)


def test_recipe_statistics():
    w = scaled(CONFIGS["cfg2_7b_32k"], n_frames=24, tokens_per_frame=64)
    q, k, v, qw = make_layer(w)
    assert q.dtype == torch.bfloat16
    d = w.head_dim
    v64 = to_f64(v).reshape(w.n_frames, w.tokens_per_frame, w.n_kv_heads, d) * math.sqrt(d)
    # frame-to-frame correlation of the AR(1) recipe: a / sqrt(a^2 var + b^2) settles near 0.9
    a, b = v64[10:-1].ravel(), v64[11:].ravel()
    corr = np.corrcoef(a, b)[0, 1]
    assert 0.85 < corr < 0.95
    # per-token log-normal key scale, shared by heads: log-norm spread of K exceeds that of V
    kn = np.log(np.linalg.norm(to_f64(k), axis=2))
    vn = np.log(np.linalg.norm(to_f64(v), axis=2))
    assert kn.std() > 0.4 and vn.std() < 0.2
    assert np.corrcoef(kn[:, 0], kn[:, 1])[0, 1] > 0.9
    # bf16 values widen exactly
    assert np.array_equal(to_f64(q).astype(np.float32), q.float().numpy())


def test_frame_recursion_summed_by_doubling_equals_the_sequential_recursion():
    # the generator sums x[f] = a x[f-1] + b eps[f] by doubling; same innovations, sequential recursion, same values
    import torch
    from paper_2505_16175_amd import workload as W
    a, b, frames = 0.9, 0.44, 37                                  # not a power of two
    x = W._ar1(torch.Generator().manual_seed(3), frames, 3, 2, 4, a, b, "cpu").view(frames, 3, 2, 4)
    eps = torch.randn(frames, 3, 2, 4, generator=torch.Generator().manual_seed(3))
    ref = torch.empty_like(eps)
    ref[0] = eps[0]
    for f in range(1, frames):
        ref[f] = a * ref[f - 1] + b * eps[f]
    assert (x - ref).abs().max() < 1e-5
