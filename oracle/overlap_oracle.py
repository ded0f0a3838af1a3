"""Oracle for the run time of the loader / prefill pipeline (Sec. 3.3 of the paper, "Overlapping ...").

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. Only the tests and the benchmark's reporting may import it; it
shares no code with the HIP library.

Sec. 3.3 describes a producer/consumer pipeline: the loader makes the frames of group after group available in
order; the prefill of a group starts as soon as its frames are there and the previous group's prefill has
finished; the GPU idles only while it waits for the loader. Two functions:

  * overlap_total    the paper's closed form (the equation of Sec. 3.3):
                         t_total = max(t_dec + t^g_prefill, t_prefill + t^g_dec) + Delta
                     with t_dec / t_prefill the total loading / prefill time, t^g_dec the time to load the first
                     group and t^g_prefill the time to prefill the last one.
  * pipeline_finish  the pipeline itself, stepped group by group from per-group availability times and per-group
                     prefill times (the definition the closed form summarises).

Reading: the closed form is exact when the critical path runs through the first group (prefill-bound: the GPU never
waits after the first group) or through the last one (loader-bound: every group is prefilled before the next
arrives); in between it is a lower bound of the stepped pipeline, which the pins check.
"""
from __future__ import annotations


def sequential_total(t_dec: float, t_prefill: float) -> float:
    """Run time without overlap (Sec. 3.3: load everything, then prefill everything)."""
    return t_dec + t_prefill


def overlap_total(t_dec: float, t_prefill: float, t_first_dec: float, t_last_prefill: float, delta: float = 0.0) -> float:
    """The equation of Sec. 3.3."""
    return max(t_dec + t_last_prefill, t_prefill + t_first_dec) + delta


def pipeline_finish(ready_times, prefill_times, delta: float = 0.0) -> float:
    """Finish time of the pipeline: group g starts at max(its availability time, the end of group g-1) and
    takes prefill_times[g]. ready_times are measured from the start of the run and must not decrease."""
    assert len(ready_times) == len(prefill_times) and len(ready_times) > 0
    end = 0.0
    prev = float("-inf")
    for ready, dur in zip(ready_times, prefill_times):
        assert ready >= prev and dur >= 0.0
        prev = ready
        start = ready if ready > end else end
        end = start + dur
    return end + delta
