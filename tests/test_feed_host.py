"""The feed's queue (include/qp_feed.h) on the host: ordering, back-pressure, closing, time-outs, argument errors.
Pageable slots, no GPU call."""
import ctypes
import threading
import time

import pytest

from paper_2505_16175_amd import binding as B


def _write(feed, payload: bytes):
    p = feed.begin_write()
    ctypes.memmove(p, payload, len(payload))
    feed.publish(len(payload))


def _read(ptr, n):
    return ctypes.string_at(ptr, n)


def test_groups_come_out_in_order_with_their_sizes():
    feed = B.Feed(3, 64, B.QP_FEED_PAGEABLE)
    try:
        msgs = [bytes([i]) * (i + 1) for i in range(3)]
        for m in msgs:
            _write(feed, m)
        for i, m in enumerate(msgs):
            st, p, n, g = feed.next(0)
            assert (st, n, g) == (B.QP_OK, len(m), i) and _read(p, n) == m
        assert feed.next(10)[0] == B.QP_FEED_TIMEOUT          # nothing published, not closed
        for i in range(3):
            feed.release(i)
        feed.close()
        assert feed.next(-1)[0] == B.QP_FEED_END
    finally:
        feed.destroy()


def test_producer_blocks_while_the_ring_is_full_and_resumes_on_release():
    feed = B.Feed(2, 16, B.QP_FEED_PAGEABLE)
    try:
        produced = []

        def producer():
            for i in range(5):
                _write(feed, bytes([i]) * 4)
                produced.append(i)
            feed.close()

        t = threading.Thread(target=producer)
        t.start()
        time.sleep(0.3)
        assert produced == [0, 1]                              # the third write waits for a free slot
        got = []
        while True:
            st, p, n, g = feed.next(-1)
            if st == B.QP_FEED_END:
                break
            got.append((g, _read(p, n)))
            feed.release(g)                                    # hands the slot back: the producer moves on
        t.join(5)
        assert not t.is_alive()
        assert got == [(i, bytes([i]) * 4) for i in range(5)]
    finally:
        feed.destroy()


def test_consumer_blocks_until_published_and_ends_after_close():
    feed = B.Feed(2, 16, B.QP_FEED_PAGEABLE)
    try:
        def late():
            time.sleep(0.15)
            _write(feed, b"xy")
            feed.close()

        t = threading.Thread(target=late)
        t0 = time.perf_counter()
        t.start()
        st, p, n, g = feed.next(-1)
        assert time.perf_counter() - t0 >= 0.14 and (st, n, g) == (B.QP_OK, 2, 0) and _read(p, n) == b"xy"
        feed.release(0)
        assert feed.next(-1)[0] == B.QP_FEED_END
        t.join()
    finally:
        feed.destroy()


def _returns_within(fn, seconds):
    t = threading.Thread(target=fn, daemon=True)
    t.start()
    t.join(seconds)
    return not t.is_alive()


def test_destroy_returns_when_the_consumer_stopped_early_with_the_ring_full():
    # the consumer gives up at group 1 of 8 with 2 slots: the stand-in producer is blocked on the full ring and
    # destroy must wake it before joining its thread
    import torch
    src = torch.arange(8 * 16, dtype=torch.uint8)
    feed = B.Feed(2, 16, B.QP_FEED_PAGEABLE)
    feed.stub_producer(src, [16] * 8, 0, 0)
    st, _, _, g = feed.next(-1)
    assert (st, g) == (B.QP_OK, 0)
    feed.release(0)
    st, _, _, g = feed.next(-1)
    assert (st, g) == (B.QP_OK, 1)                             # never released: the consumer "fails" here
    time.sleep(0.2)                                            # the producer has filled the ring and is waiting
    assert _returns_within(feed.destroy, 5.0)


def test_stop_wakes_a_blocked_producer_and_refuses_later_writes():
    feed = B.Feed(2, 16, B.QP_FEED_PAGEABLE)
    try:
        _write(feed, b"a")
        _write(feed, b"b")
        seen = []

        def third():
            try:
                _write(feed, b"c")
                seen.append("written")
            except B.QPError as e:
                seen.append(e.status)

        t = threading.Thread(target=third, daemon=True)
        t.start()
        time.sleep(0.2)
        assert seen == []                                      # blocked: both slots are published and unreleased
        feed.stop()
        t.join(5)
        assert seen == [B.QP_FEED_END]
        with pytest.raises(B.QPError) as e:
            feed.begin_write()
        assert e.value.status == B.QP_FEED_END
        assert feed.next(0)[0] == B.QP_OK                      # what was published can still be taken
    finally:
        feed.destroy()


def test_stub_producer_paces_the_groups():
    import torch
    feed = B.Feed(2, 8, B.QP_FEED_PAGEABLE)
    try:
        src = torch.arange(24, dtype=torch.uint8)
        feed.stub_producer(src, [8, 8, 8], 100_000, 50_000)     # due at 100, 150, 200 ms
        t0 = time.perf_counter()
        due = []
        while True:
            st, p, n, g = feed.next(-1)
            if st == B.QP_FEED_END:
                break
            due.append(time.perf_counter() - t0)
            assert _read(p, n) == bytes(range(8 * g, 8 * g + 8))
            feed.release(g)
        ms = feed.stub_join()
        # never early; the upper bounds leave room for a busy host
        assert len(due) == 3 and 0.099 < due[0] < 0.4 and 0.149 < due[1] < 0.45 and 0.199 < due[2] < 0.5
        assert 199 < ms < 500
    finally:
        feed.destroy()


def test_argument_errors():
    with pytest.raises(B.QPError):
        B.Feed(1, 16, B.QP_FEED_PAGEABLE)                      # at least two slots
    with pytest.raises(B.QPError):
        B.Feed(2, 0, B.QP_FEED_PAGEABLE)
    feed = B.Feed(2, 4, B.QP_FEED_PAGEABLE)
    try:
        with pytest.raises(B.QPError):
            feed.publish(1)                                    # no slot obtained
        feed.begin_write()
        with pytest.raises(B.QPError):
            feed.begin_write()                                 # the previous slot was not published
        with pytest.raises(B.QPError) as e:
            feed.publish(5)                                    # larger than a slot
        assert e.value.status == B.QP_ERR_CAPACITY
        feed.publish(4)
        with pytest.raises(B.QPError):
            feed.release(0)                                    # not taken yet
        feed.close()
        with pytest.raises(B.QPError):
            feed.begin_write()                                 # closed
    finally:
        feed.destroy()


@pytest.mark.parametrize("n_slots", [2, 3, 5])
def test_queue_under_random_pacing(n_slots):
    """Many groups through a small ring with a producer and a consumer that stall at random: nothing is lost,
    duplicated, reordered or overwritten while in use, and both sides terminate."""
    import random
    import struct
    n_groups = 400
    feed = B.Feed(n_slots, 64, B.QP_FEED_PAGEABLE)
    rng_p, rng_c = random.Random(1), random.Random(2)
    errors = []

    def producer():
        try:
            for i in range(n_groups):
                if rng_p.random() < 0.1:
                    time.sleep(rng_p.random() * 0.002)
                size = 8 + (i % 7) * 8
                _write(feed, struct.pack("<q", i) * (size // 8))
            feed.close()
        except Exception as e:   # noqa: BLE001
            errors.append(e)

    t = threading.Thread(target=producer)
    t.start()
    held, seen = [], []
    try:
        while True:
            st, p, n, g = feed.next(2000)
            assert st != B.QP_FEED_TIMEOUT, "consumer starved: dead-lock between ring and queue"
            if st == B.QP_FEED_END:
                break
            held.append((g, p, n))
            if rng_c.random() < 0.1:
                time.sleep(rng_c.random() * 0.002)
            # keep up to n_slots - 1 groups in hand, check them when they are handed back (not overwritten meanwhile)
            while len(held) > rng_c.randrange(0, n_slots):
                g0, p0, n0 = held.pop(0)
                assert n0 == 8 + (g0 % 7) * 8 and _read(p0, n0) == struct.pack("<q", g0) * (n0 // 8)
                seen.append(g0)
                feed.release(g0)
        for g0, p0, n0 in held:
            assert _read(p0, n0) == struct.pack("<q", g0) * (n0 // 8)
            seen.append(g0)
            feed.release(g0)
        t.join(10)
        assert not t.is_alive() and not errors
        assert seen == list(range(n_groups))
    finally:
        feed.close()
        t.join(10)
        feed.destroy()
