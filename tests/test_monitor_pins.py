"""Pins for the online-monitor oracle (CPU only; nothing here calls the C++ implementation)."""
import math

import pytest

from oracle import monitor as M


def test_hand_worked_trace():
    # W = 1.  Window 0: two requests, L_req = (2 + 4)/2 = 3, L_exec = (2 + 2)/2 = 2, ratio 1.5 -> not above 1.5
    # Window 1: empty -> policy stays.  Window 2: ratio 5/2 = 2.5 -> throughput.  Window 3: ratio 1 -> latency.
    reqs = [(0.2, 2.0, 2.0), (0.9, 4.0, 2.0), (2.5, 5.0, 2.0), (3.0, 1.0, 1.0), (3.999, 3.0, 3.0)]
    got = M.monitor_run(reqs, W=1.0, beta=1.5, t_end=4.0)
    assert [g[0] for g in got] == [0, 1, 2, 3]
    assert got[0][1] == pytest.approx(1.5) and got[0][2] == M.LATENCY
    assert math.isnan(got[1][1]) and got[1][2] == M.LATENCY
    assert got[2][1] == pytest.approx(2.5) and got[2][2] == M.THROUGHPUT
    assert got[3][1] == pytest.approx(1.0) and got[3][2] == M.LATENCY
    assert M.switch_count(got) == 2
    # ratio of means, not mean of ratios: (1 + 9)/(1 + 1) = 5 vs mean(1, 9) = 5 -- choose a case that differs
    got = M.monitor_run([(0.1, 1.0, 1.0), (0.2, 9.0, 3.0)], W=1.0, beta=2.2, t_end=1.0)
    assert got[0][1] == pytest.approx(10.0 / 4.0)          # mean of ratios would be 2.0
    assert got[0][2] == M.THROUGHPUT


def test_exec_latency_adds_groups_and_communication():
    assert M.exec_latency([0.25, 0.5, 0.125], 0.0625) == 0.9375


def deterministic_queue(n, arrival_gap, service):
    """Single server, arrivals every `arrival_gap`, constant service time: request i waits
    max(0, i * (service - arrival_gap))."""
    out, free = [], 0.0
    for i in range(n):
        arrive = i * arrival_gap
        start = max(arrive, free)
        free = start + service
        out.append((free, free - arrive, service))
    return out


def test_underloaded_queue_never_leaves_the_latency_policy():
    reqs = deterministic_queue(200, arrival_gap=0.05, service=0.04)
    got = M.monitor_run(reqs, W=0.3, beta=1.5)
    assert got and all(r == pytest.approx(1.0) and p == M.LATENCY for (_, r, p) in got)


def test_overloaded_queue_crosses_the_threshold_where_the_closed_form_says():
    gap, s = 3 / 64, 1 / 16                  # binary fractions: every time below is exact; request i waits i / 64
    reqs = deterministic_queue(400, gap, s)
    got = M.monitor_run(reqs, W=0.5, beta=1.5)
    for (n, ratio, policy) in got:
        idx = [i for i in range(400) if n * 0.5 <= (i + 1) * s < (n + 1) * 0.5]     # completes at (i+1) s
        want = 1.0 + sum(i * (s - gap) for i in idx) / len(idx) / s
        assert ratio == pytest.approx(want)
        assert policy == (M.THROUGHPUT if want > 1.5 else M.LATENCY)
    assert got[0][2] == M.LATENCY or got[0][1] > 1.5
    assert got[-1][2] == M.THROUGHPUT and M.switch_count(got) == 1


def test_threshold_limits_and_time_unit_invariance():
    reqs = deterministic_queue(300, 3 / 64, 1 / 16)
    assert all(p == M.LATENCY for (_, _, p) in M.monitor_run(reqs, 0.3, beta=1e9))
    got = M.monitor_run(reqs[1:], 0.25, beta=1.0)                       # every request but the first waited
    assert all(p == M.THROUGHPUT for (_, r, p) in got if not math.isnan(r)) and got[0][2] == M.THROUGHPUT
    a = M.monitor_run(reqs, 0.25, 1.5)
    scaled = [(1024 * t, 1024 * lr, 1024 * le) for (t, lr, le) in reqs]
    b = M.monitor_run(scaled, 256.0, 1.5)
    assert [(n, p) for (n, _, p) in a] == [(n, p) for (n, _, p) in b]
    assert [r for (_, r, _) in a] == pytest.approx([r for (_, r, _) in b])


def test_window_membership_is_half_open():
    got = M.monitor_run([(1.0, 4.0, 1.0)], W=1.0, beta=1.5, t_end=2.0)
    assert math.isnan(got[0][1]) and got[1][1] == pytest.approx(4.0)
