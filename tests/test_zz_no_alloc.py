"""qp_group_attend_noalloc (the entry point for callers that cannot allocate: its scratch is a device array the
library holds) against qp_group_attend with a caller workspace of the same size: same launch layout, same bits."""
import numpy as np
import pytest
import torch

from helpers import assert_attn_close
from oracle import qp_oracle as O
from paper_2505_16175_amd import binding as B
from paper_2505_16175_amd.workload import to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _inputs(n_g, h_q, h_kv, c, seed):
    g = torch.Generator().manual_seed(seed)
    bf = lambda *s: torch.randn(*s, generator=g).to(torch.bfloat16)
    return bf(n_g, h_q, 128), bf(n_g, h_kv, 128), bf(n_g, h_kv, 128), bf(h_kv, c, 128), bf(h_kv, c, 128)


def test_noalloc_equals_the_workspace_entry_point_on_two_calls_in_a_row():
    h_q, h_kv, c = 28, 4, 5000
    layout = B.make_layout(h_q, h_kv, 128, "bf16")
    ws = torch.empty(B.NOALLOC_SCRATCH_BYTES, dtype=torch.uint8, device=DEV)
    assert ws.data_ptr() % 256 == 0
    for n_g, seed in ((64, 1), (1, 2), (7, 3)):                 # a text chunk, then smaller inputs: decode, a short chunk
        print(f"case n_g={n_g}", flush=True)
        q, k, v, ck, cv = _inputs(n_g, h_q, h_kv, c, seed)
        cache = B.Cache(layout, c)
        cache.k.copy_(ck)
        cache.v.copy_(cv)
        cache.c.len = c
        plan = B.attend_plan(layout, n_g, c, B.NOALLOC_SCRATCH_BYTES)
        assert plan["key_chunks"] > 1 and 0 < plan["scratch_bytes"] <= B.NOALLOC_SCRATCH_BYTES   # the scratch is in use
        dq, dk, dv = q.to(DEV), k.to(DEV), v.to(DEV)
        want = torch.full_like(dq, float("nan"))
        want_lse = torch.full((h_q, n_g), float("nan"), dtype=torch.float32, device=DEV)
        B.group_attend(layout, dq, dk, dv, cache, want, want_lse, ws)
        got = torch.full_like(dq, float("nan"))
        got_lse = torch.full_like(want_lse, float("nan"))
        B.group_attend_noalloc(layout, dq, dk, dv, cache, got, got_lse)
        torch.cuda.synchronize()
        assert torch.equal(got, want) and torch.equal(got_lse, want_lse)
        ref, ref_lse = O.attend_group(to_f64(q), to_f64(k), to_f64(v), to_f64(ck), to_f64(cv), return_lse=True)
        assert_attn_close(to_f64(got), ref, "bf16", f"noalloc n_g={n_g}")
        np.testing.assert_allclose(to_f64(got_lse), ref_lse, atol=2e-3)


def test_noalloc_rejects_sizes_beyond_its_limit_and_bad_arguments():
    layout = B.make_layout(28, 4, 128, "bf16")
    n_g = B.NOALLOC_MAX_ROWS // 28 + 1
    q, k, v, ck, cv = _inputs(n_g, 28, 4, 64, 9)
    cache = B.Cache(layout, 64)
    cache.c.len = 64
    out = torch.empty_like(q, device=DEV)
    with pytest.raises(B.QPError) as e:
        B.group_attend_noalloc(layout, q.to(DEV), k.to(DEV), v.to(DEV), cache, out)
    assert e.value.status == B.QP_ERR_CAPACITY
    with pytest.raises(B.QPError) as e:
        B.group_attend_noalloc(layout, q.to(DEV)[:1], None, v.to(DEV)[:1], cache, out[:1])
    assert e.value.status == B.QP_ERR_INVALID_ARG
