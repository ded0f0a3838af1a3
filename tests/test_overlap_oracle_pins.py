"""Pins for oracle/overlap_oracle.py (Sec. 3.3's run-time equation and the pipeline it summarises). CPU only."""
import itertools

import numpy as np
import pytest

from oracle import overlap_oracle as oo


def test_equation_hand_cases_both_regimes_and_the_crossover():
    # loader-bound: loading 100, prefill 30, first group loaded after 10, last group prefilled in 4 -> 100 + 4
    assert oo.overlap_total(100.0, 30.0, 10.0, 4.0) == 104.0
    # prefill-bound: loading 20, prefill 90, first group after 2.5, last group 12 -> 90 + 2.5
    assert oo.overlap_total(20.0, 90.0, 2.5, 12.0) == 92.5
    # crossover: both arguments of the max equal
    assert oo.overlap_total(50.0, 40.0, 15.0, 5.0) == 55.0
    # delta is added after the max, once
    assert oo.overlap_total(100.0, 30.0, 10.0, 4.0, delta=2.8) == pytest.approx(106.8)
    assert oo.sequential_total(49.7, 20.0) == pytest.approx(69.7)


def test_equation_with_one_group_is_the_sequential_time():
    # a single group: its loading is all the loading, its prefill all the prefill; nothing can overlap
    assert oo.overlap_total(7.0, 3.0, 7.0, 3.0) == oo.sequential_total(7.0, 3.0) == 10.0


def test_equation_never_exceeds_sequential_and_never_beats_either_stage():
    rng = np.random.default_rng(5)
    for _ in range(200):
        t_dec, t_pre = rng.uniform(1, 100, 2)
        t_fd, t_lp = rng.uniform(0, 1) * t_dec, rng.uniform(0, 1) * t_pre
        t = oo.overlap_total(t_dec, t_pre, t_fd, t_lp)
        assert max(t_dec, t_pre) <= t <= oo.sequential_total(t_dec, t_pre) + 1e-12


def test_pipeline_by_hand():
    # groups ready at 1, 2, 10; prefill 3, 3, 3: g0 runs 1-4, g1 4-7, g2 waits for the loader: 10-13
    assert oo.pipeline_finish([1.0, 2.0, 10.0], [3.0, 3.0, 3.0]) == 13.0
    # same loader, slow prefill: 1-6, 6-11, 11-16
    assert oo.pipeline_finish([1.0, 2.0, 10.0], [5.0, 5.0, 5.0]) == 16.0
    assert oo.pipeline_finish([4.0], [2.5], delta=0.5) == 7.0


def test_pipeline_equals_brute_force_over_critical_groups():
    # the finish time is the longest chain "wait for group j, then prefill j..G-1 back to back"
    rng = np.random.default_rng(11)
    for _ in range(100):
        g = int(rng.integers(1, 9))
        ready = np.cumsum(rng.uniform(0, 5, g))
        dur = rng.uniform(0, 5, g)
        want = max(ready[j] + dur[j:].sum() for j in range(g))
        assert oo.pipeline_finish(list(ready), list(dur)) == pytest.approx(want, rel=1e-14)


@pytest.mark.parametrize("first,per,dur", [(12.0, 12.0, 4.6), (3.0, 0.5, 4.6), (5.0, 6.0, 6.0), (0.0, 1.0, 1.0)])
def test_equation_is_exact_for_a_steady_loader_and_equal_groups(first, per, dur):
    # steady loader (first group after `first`, one more every `per`) and equal prefill times: the critical path
    # goes through the first or the last group, so the closed form equals the stepped pipeline
    g = 8
    ready = [first + i * per for i in range(g)]
    t_dec, t_pre = ready[-1], g * dur
    assert oo.pipeline_finish(ready, [dur] * g) == pytest.approx(oo.overlap_total(t_dec, t_pre, first, dur), rel=1e-14)


def test_equation_is_a_lower_bound_of_the_pipeline():
    rng = np.random.default_rng(3)
    strict = 0
    for _ in range(300):
        g = int(rng.integers(2, 10))
        ready = np.cumsum(rng.uniform(0, 5, g))
        dur = rng.uniform(0.1, 5, g)
        eq = oo.overlap_total(ready[-1], dur.sum(), ready[0], dur[-1])
        sim = oo.pipeline_finish(list(ready), list(dur))
        assert sim >= eq - 1e-12
        assert sim <= oo.sequential_total(ready[-1], dur.sum()) + 1e-12
        strict += sim > eq + 1e-9
    assert strict > 0                                          # a critical group in the middle does occur
