"""Pins for the dynamic-offloading oracle (paper section 5.3)."""
import numpy as np

from oracle.offload_window import INIT, IN_PROGRESS, STEADY, OffloadWindowOracle


def test_the_sections_worked_example():
    # "if only one page is duplicated and an inference query requires three pages, the query
    # must wait until the current and end pointers advance by two additional pages"
    w = OffloadWindowOracle(window=1)
    for p in range(10):
        w.release(p)
    assert (w.start, w.current, w.end) == (0, 0, 1) and w.state() == INIT
    w.offloaded(1)
    assert w.state() == STEADY and (w.current, w.end) == (1, 1)
    assert w.take(3) is None                       # stalls ...
    assert w.end == 3 and w.current == 1           # ... end has moved by two, current must follow
    w.offloaded(1)
    assert w.take(3) is None and w.state() == IN_PROGRESS
    w.offloaded(1)
    assert w.take(3) == [0, 1, 2]
    # "if three pages are duplicated, the same query can proceed immediately"
    w = OffloadWindowOracle(window=3)
    for p in range(10):
        w.release(p)
    w.offloaded(3)
    assert w.take(3) == [0, 1, 2]
    # state 3: the end pointer moved forward by the number of pages taken
    assert (w.start, w.current, w.end) == (3, 3, 6) and w.state() == INIT


def test_four_states_in_order():
    w = OffloadWindowOracle(window=4)
    assert w.state() == STEADY                     # nothing scheduled
    for p in range(6):
        w.release(100 + p)
    assert w.state() == INIT and w.scheduled() == [100, 101, 102, 103]
    w.offloaded(2)
    assert w.state() == IN_PROGRESS and w.scheduled() == [102, 103]
    assert w.take(2) == [100, 101]                 # query arrival
    assert (w.start, w.current, w.end) == (2, 2, 6) and w.scheduled() == [102, 103, 104, 105]
    w.offloaded(4)
    assert w.state() == STEADY
    assert w.take(5) is None and w.take(4) == [102, 103, 104, 105]
    assert w.take(1) is None                       # no free page left


def test_invariants_under_random_operations():
    rng = np.random.default_rng(0)
    for window in (1, 2, 5, 16):
        w = OffloadWindowOracle(window)
        nxt, taken = 0, []
        for _ in range(3000):
            op = rng.integers(0, 3)
            if op == 0:
                for _ in range(rng.integers(1, 6)):
                    w.release(nxt)
                    nxt += 1
            elif op == 1 and w.scheduled():
                w.offloaded(int(rng.integers(1, len(w.scheduled()) + 1)))
            elif op == 2:
                n = int(rng.integers(1, 8))
                before = (w.start, w.current)
                got = w.take(n)
                if got is None:
                    assert n > before[1] - before[0]            # it was not covered
                    assert w.start == before[0]
                else:
                    assert n <= before[1] - before[0]
                    taken += got
            assert 0 <= w.start <= w.current <= w.end <= w.tail
            # the window is kept when there are enough free pages
            assert w.end - w.start >= min(window, w.tail - w.start) or w.end == w.tail
        assert taken == list(range(len(taken)))                  # pages leave in queue order, once
