"""Comparison helpers shared by the GPU parity tests (no method arithmetic of their own)."""
import numpy as np

from paper_2505_16175_amd.workload import to_f64

# Tolerances of the benchmark definition: bf16 outputs within 2e-2 absolute / 1e-2 relative of the
# fp64 oracle, f32 within 1e-5. |O| is small under the literal 1/sqrt(d) input scaling, so a
# normalised-error gate is applied as well (a wrong kernel must not pass on the absolute term).
TOL = {"bf16": dict(atol=2e-2, rtol=1e-2, nrm=1e-2), "f32": dict(atol=1e-5, rtol=1e-5, nrm=1e-5)}
NEAR_TIE_REL_GAP = 1e-5


def assert_attn_close(got, want, dtype, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    t = TOL[dtype]
    err = np.abs(got - want)
    bad = err > t["atol"] + t["rtol"] * np.abs(want)
    nrm = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    assert not bad.any(), f"{what}: {bad.sum()} elements out of tolerance, max abs err {err.max():.3e}"
    assert nrm <= t["nrm"], f"{what}: normalised error {nrm:.3e} > {t['nrm']}"
    return dict(max_abs=float(err.max()), nrm=float(nrm))


def compare_kept(got_idx, want_idx, oracle_scores):
    """Exact kept-set parity per head, except near-ties (relative score gap < 1e-5), which are counted.

    got_idx / want_idx: [H, k] ascending; oracle_scores: [H, n] float64.
    Returns the number of excused (near-tie) heads; raises on any other mismatch.
    """
    got_idx = np.asarray(got_idx)
    want_idx = np.asarray(want_idx)
    assert got_idx.shape == want_idx.shape, (got_idx.shape, want_idx.shape)
    excused = 0
    for h in range(got_idx.shape[0]):
        g, w = got_idx[h], want_idx[h]
        assert (np.diff(g) > 0).all(), f"head {h}: kept indices not strictly ascending"
        assert g.min() >= 0 and g.max() < oracle_scores.shape[1], f"head {h}: kept index out of range"
        if (g == w).all():
            continue
        diff = np.setxor1d(g, w)
        s_k = np.sort(oracle_scores[h])[::-1][len(w) - 1]          # k-th largest oracle score
        gap = np.abs(oracle_scores[h][diff] - s_k)
        assert (gap < NEAR_TIE_REL_GAP * abs(s_k)).all(), \
            f"head {h}: kept sets differ at {diff.tolist()} beyond a near-tie (gaps {gap.tolist()}, s_k {s_k})"
        excused += 1
    return excused


def sample_rows(n_g, n_samples, rng, tile=32):
    """Group-token rows to check: first, last, both sides of some tile boundaries, and random ones."""
    rows = {0, n_g - 1}
    for b in (tile, 2 * tile, 128, 256, n_g // 2, n_g - tile):
        for r in (b - 1, b):
            if 0 <= r < n_g:
                rows.add(r)
    while len(rows) < min(n_g, n_samples):
        rows.add(int(rng.integers(0, n_g)))
    return sorted(rows)


# ---- the decoder layer around the path: the product's fused weight tensors split into the layer oracle's names ----
def oracle_weights(w, dims):
    hq, hkv = dims.n_q_heads * 128, dims.n_kv_heads * 128
    f = {k: to_f64(v) for k, v in w.items()}
    return dict(ln1=f["ln1_w"], ln2=f["ln2_w"], w_q=f["w_qkv"][:hq], b_q=f["b_qkv"][:hq],
                w_k=f["w_qkv"][hq:hq + hkv], b_k=f["b_qkv"][hq:hq + hkv], w_v=f["w_qkv"][hq + hkv:],
                b_v=f["b_qkv"][hq + hkv:], w_o=f["w_o"], w_gate=f["w_gate_up"][:dims.d_ff],
                w_up=f["w_gate_up"][dims.d_ff:], w_down=f["w_down"])


def oracle_shape(dims):
    return dict(n_q_heads=dims.n_q_heads, n_kv_heads=dims.n_kv_heads, head_dim=128, d_model=dims.d_model,
                rms_eps=dims.rms_eps, rope_theta=dims.rope_theta, mrope_section=dims.mrope_section)


# Through a whole layer the attention kernel's own tolerance applies (it rounds the softmax numerators to bf16:
# up to 2e-2 absolute / 1e-2 relative on the attention output), carried through W_o and the MLP; everything else
# is one-ulp rounding flips. Layers add their errors, so the absolute floor grows with the depth of the stack;
# the normalised error stays under the attention kernel's 1e-2. A wrong operand, index or epilogue gives errors
# of the size of the RMS itself.
def assert_layer_close(got, want, what, layers=1):
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    rms = np.sqrt(np.mean(want * want))
    err = np.abs(got - want)
    rel = np.linalg.norm(got - want) / np.linalg.norm(want)
    print(f"{what}: normalised error {rel:.2e}, max abs error {err.max():.2e}, rms {rms:.2e}", flush=True)
    bad = err > 2e-2 * np.abs(want) + 2e-2 * layers * rms
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} out of tolerance, max err {err.max():.3e} (rms {rms:.3e})"
    assert rel <= 1e-2, f"{what}: normalised error {rel:.3e}"
    return rel
