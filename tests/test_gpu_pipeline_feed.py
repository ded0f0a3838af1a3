"""GPU tests of the feed (include/qp_feed.h): a stack fed group by group from the host equals the layer oracle's
stack and, bit for bit, the same stack driven directly; the run time follows the oracle's pipeline model and the
equation of Sec. 3.3."""
import time

import numpy as np
import pytest
import torch

from helpers import assert_layer_close, oracle_shape, oracle_weights
from oracle import layer_oracle as LO
from oracle import overlap_oracle as OO
from oracle import qp_oracle as O
from paper_2505_16175_amd import binding as B
from paper_2505_16175_amd import workload as W
from paper_2505_16175_amd.workload import to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda"


class Stack:
    """A few decoder layers around the path, driven group by group (the group-major schedule of Sec. 3.2)."""

    def __init__(self, dims, n_layers, bounds, retention, rule="key_norm_small", shared_weights=False):
        self.dims, self.bounds, self.retention, self.rule = dims, bounds, retention, rule
        self.layout = B.make_layout(dims.n_q_heads, dims.n_kv_heads, 128, "bf16")
        self.shape = B.make_layer_shape(dims.d_model, dims.d_ff, dims.rms_eps, dims.rope_theta, dims.mrope_section)
        first = B.LayerWeights(**W.make_decoder_layer(dims, 0, device=DEV))
        self.weights = [first if shared_weights else B.LayerWeights(**W.make_decoder_layer(dims, l, device=DEV))
                        for l in range(n_layers)] if not shared_weights else [first] * n_layers
        self.n_max = max(n for _, n in bounds)
        self.ws = B.make_layer_workspace(self.layout, self.shape, self.n_max, 0)
        cap = sum(B.keep_count(n, retention) for _, n in bounds)
        self.caches = [B.Cache(self.layout, cap) for _ in range(n_layers)]
        n_tok = bounds[-1][0] + bounds[-1][1]
        self.pos = W.video_positions((n_tok + 15) // 16, 16, device=DEV)[:, :n_tok].contiguous()
        self.out = torch.zeros(n_tok, dims.d_model, dtype=torch.bfloat16, device=DEV)
        self.tmp = [torch.empty(self.n_max, dims.d_model, dtype=torch.bfloat16, device=DEV) for _ in range(2)]

    def reset(self):
        for c in self.caches:
            c.reset()
        self.out.zero_()

    def group(self, g, x_g):
        base, n_g = self.bounds[g]
        keep = B.keep_count(n_g, self.retention)
        cur = x_g
        for l, wt in enumerate(self.weights):
            nxt = self.out[base:base + n_g] if l == len(self.weights) - 1 else self.tmp[l & 1][:n_g]
            B.layer_group(self.layout, self.shape, wt, cur, self.pos, base, base, None, self.rule, keep, self.caches[l],
                          nxt, None, self.ws)
            cur = nxt


def _consume(stack, feed, d_model):
    bufs = [torch.empty(stack.n_max, d_model, dtype=torch.bfloat16, device=DEV) for _ in range(2)]

    def fn(group, dev_ptr, nbytes):
        buf = bufs[0] if dev_ptr == bufs[0].data_ptr() else bufs[1]
        assert dev_ptr == buf.data_ptr() and nbytes == stack.bounds[group][1] * d_model * 2
        stack.group(group, buf[:stack.bounds[group][1]])

    return feed.consume(bufs[0], bufs[1], fn)


def test_fed_stack_equals_direct_stack():
    dims = W.LayerDims(256, 384, 4, 2)
    frames, tpf, gf = 11, 36, 3                                  # ragged last group
    bounds = O.group_bounds(frames, tpf, gf)
    x = W.make_hidden(frames, tpf, dims.d_model)
    stack = Stack(dims, 2, bounds, 0.4)
    xd = x.to(DEV)
    for g, (base, n_g) in enumerate(bounds):
        stack.group(g, xd[base:base + n_g])
    torch.cuda.synchronize()
    want = stack.out.clone()
    want_caches = [(c.k.clone(), c.v.clone(), c.pos.clone(), c.len) for c in stack.caches]
    for slots in (2, 3):
        stack.reset()
        feed = B.Feed(slots, stack.n_max * dims.d_model * 2)
        try:
            feed.stub_producer(x, [n * dims.d_model * 2 for _, n in bounds], 2000, 500)
            stats = _consume(stack, feed, dims.d_model)
            feed.stub_join()
        finally:
            feed.destroy()
        assert stats["groups"] == len(bounds)
        assert torch.equal(stack.out, want)
        for c, (k, v, p, n) in zip(stack.caches, want_caches):
            assert c.len == n and torch.equal(c.k, k) and torch.equal(c.v, v) and torch.equal(c.pos, p)


def test_fed_stack_matches_the_layer_oracle():
    """The fed run against the fp64 layer oracle (not against another GPU run): two layers, four groups with a
    ragged last one, nothing pruned, so that no selection decision enters; outputs, cache rows and positions."""
    dims = W.LayerDims(256, 384, 4, 2)
    frames, tpf, gf = 11, 36, 3
    bounds = O.group_bounds(frames, tpf, gf)
    x = W.make_hidden(frames, tpf, dims.d_model)
    stack = Stack(dims, 2, bounds, 1.0)
    feed = B.Feed(2, stack.n_max * dims.d_model * 2)
    try:
        feed.stub_producer(x, [n * dims.d_model * 2 for _, n in bounds], 1000, 300)
        stats = _consume(stack, feed, dims.d_model)
        feed.stub_join()
    finally:
        feed.destroy()
    assert stats["groups"] == len(bounds)
    layers = [oracle_weights(wt.tensors, dims) for wt in stack.weights]          # generated on the GPU: read them back
    want, want_caches = LO.layer_stack(to_f64(x), stack.pos.cpu().numpy(), layers, oracle_shape(dims), bounds, None, None,
                                       "key_norm_small", 1.0, store=LO.bf16_round)
    assert_layer_close(to_f64(stack.out), want, "fed stack output", layers=2)
    for l, (cache, (ck, cv, cp)) in enumerate(zip(stack.caches, want_caches)):
        assert cache.len == frames * tpf
        np.testing.assert_array_equal(cache.pos.cpu().numpy()[:, :cache.len], cp)
        assert_layer_close(to_f64(cache.k)[:, :cache.len], ck, f"layer {l} cached K", layers=l + 1)
        assert_layer_close(to_f64(cache.v)[:, :cache.len], cv, f"layer {l} cached V", layers=l + 1)


def test_consumer_that_fails_early_leaves_no_blocked_producer():
    """The group function fails at group 1 of 8 with a ring of 2 slots: qp_feed_consume reports the failure, and the
    stand-in loader, which was waiting for a free slot, ends instead of blocking destroy for ever."""
    n_groups, nbytes = 8, 4096
    src = torch.zeros(n_groups * nbytes, dtype=torch.uint8).pin_memory()
    feed = B.Feed(2, nbytes)
    bufs = [torch.empty(nbytes, dtype=torch.uint8, device=DEV) for _ in range(2)]

    def fn(group, dev_ptr, n):
        if group == 1:
            raise B.QPError(B.QP_ERR_INVALID_ARG, "group function of the test")

    t0 = time.perf_counter()
    try:
        feed.stub_producer(src, [nbytes] * n_groups, 0, 0)
        with pytest.raises(B.QPError):
            feed.consume(bufs[0], bufs[1], fn)
        feed.stub_join()
    finally:
        feed.destroy()
    assert time.perf_counter() - t0 < 10.0


def test_group_larger_than_the_device_buffer_is_refused():
    feed = B.Feed(2, 1024)
    try:
        src = torch.zeros(1024, dtype=torch.uint8)
        feed.stub_producer(src, [1024], 0, 0)
        small = [torch.empty(512, dtype=torch.uint8, device=DEV) for _ in range(2)]
        with pytest.raises(B.QPError) as e:
            feed.consume(small[0], small[1], lambda g, p, n: None)
        assert e.value.status == B.QP_ERR_CAPACITY
        feed.stub_join()
    finally:
        feed.destroy()


@pytest.mark.parametrize("first_ms,group_ms", [(12.0, 12.0), (3.0, 0.5)], ids=["loader_bound", "prefill_bound"])
def test_run_time_follows_the_overlap_equation(first_ms, group_ms):
    """Sec. 3.3: t_total = max(t_dec + t^g_prefill, t_prefill + t^g_dec) + delta. A 7B-shaped layer applied four
    times per group (about 5 ms per group of 2048 tokens), eight groups, against a loader that delivers the first
    group after first_ms and one more every group_ms."""
    dims = W.LAYER_DIMS["7b"]
    n_groups, n_g = 8, 2048
    bounds = [(g * n_g, n_g) for g in range(n_groups)]
    stack = Stack(dims, 4, bounds, 0.3, shared_weights=True)
    x = W.make_hidden(n_groups * 16, 128, dims.d_model).pin_memory()
    xd = x.to(DEV)

    def direct():
        stack.reset()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for g, (base, n) in enumerate(bounds):
            if g == n_groups - 1:
                torch.cuda.synchronize()
                t_last = time.perf_counter()
            stack.group(g, xd[base:base + n])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return (t1 - t0) * 1e3, (t1 - t_last) * 1e3

    direct()
    t_prefill, t_last_group = direct()
    t_dec = first_ms + (n_groups - 1) * group_ms
    expect = OO.overlap_total(t_dec, t_prefill, first_ms, t_last_group)
    # the pipeline stepped group by group with the loader's schedule and equal shares of the measured prefill time
    # (the last group measured on its own): the closed form is its lower bound and, for this steady loader, close to it
    per_group = [(t_prefill - t_last_group) / (n_groups - 1)] * (n_groups - 1) + [t_last_group]
    stepped = OO.pipeline_finish([first_ms + g * group_ms for g in range(n_groups)], per_group)
    assert expect - 1e-9 <= stepped <= OO.sequential_total(t_dec, t_prefill)
    stack.reset()
    torch.cuda.synchronize()
    feed = B.Feed(3, n_g * dims.d_model * 2)
    try:
        feed.stub_producer(x, [n_g * dims.d_model * 2] * n_groups, int(first_ms * 1000), int(group_ms * 1000))
        stats = _consume(stack, feed, dims.d_model)
        producer_ms = feed.stub_join()
    finally:
        feed.destroy()
    print(f"t_prefill {t_prefill:.2f} ms, last group {t_last_group:.2f} ms, t_dec {t_dec:.2f} ms (producer took "
          f"{producer_ms:.2f}); equation {expect:.2f} + delta, stepped pipeline {stepped:.2f}, measured {stats['total_ms']:.2f} ms, waited "
          f"{stats['waited_ms']:.2f} ms (first group {stats['first_group_wait_ms']:.2f})", flush=True)
    assert stats["groups"] == n_groups
    # delta: one group's host->device copy (15 MB, 0.3 ms), launch and timer slack (observed 0.7-1.5 ms; the bound
    # leaves room for a noisy host). In the loader-bound case running the two sides one after the other adds 30 ms.
    assert expect - 2.0 <= stats["total_ms"] <= expect + 12.0
    assert stepped - 2.0 <= stats["total_ms"] <= stepped + 12.0
    if OO.sequential_total(t_dec, t_prefill) - expect > 20.0:   # where overlap has something to win, it is won
        assert stats["total_ms"] < OO.sequential_total(t_dec, t_prefill) - 15.0
    assert abs(stats["first_group_wait_ms"] - first_ms) < 5.0
