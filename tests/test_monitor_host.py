"""The C++ online monitor against the oracle (host only, no GPU): same decisions window by window on
simulated single-server queues with Poisson arrivals, the load pattern of the paper's online experiments."""
import math

import numpy as np
import pytest

from oracle import monitor as M
from paper_2604_10180_amd import binding as B


def poisson_queue(rng, n, rate_fn, groups=4):
    """Single server fed by a Poisson process whose rate changes over time; each request has `groups`
    kernel-group latencies and a communication time.  Returns records sorted by completion time."""
    t, free, out = 0.0, 0.0, []
    for _ in range(n):
        t += rng.exponential(1.0 / rate_fn(t))
        g = rng.uniform(0.002, 0.006, size=groups)
        comm = float(rng.uniform(0.0005, 0.002))
        service = float(g.sum()) + comm
        start = max(t, free)
        free = start + service
        out.append((free, free - t, [float(v) for v in g], comm))
    return sorted(out, key=lambda r: r[0])


def run_product(records, W, beta, initial, t_end):
    h = B.ts_monitor_create(W, beta, initial)
    try:
        got, k, prev_closed = [], 0, 0
        n_windows = int(math.floor(t_end / W))
        for n in range(n_windows):
            while k < len(records) and records[k][0] < (n + 1) * W:
                B.ts_monitor_record(h, records[k][0], records[k][1], records[k][2], records[k][3])
                k += 1
            pol, closed, sw, ratio = B.ts_monitor_advance(h, (n + 1) * W)
            assert closed == n + 1
            got.append((pol, sw, ratio))
        return got
    finally:
        B.ts_monitor_destroy(h)


@pytest.mark.parametrize("W,beta", [(0.3, 1.5), (0.03, 1.1), (1.5, 3.0), (0.25, 1.5)])
def test_decisions_match_the_oracle_on_bursty_poisson_load(W, beta):
    rng = np.random.default_rng(int(W * 1000) + int(beta * 10))
    # light load, a burst above the service rate (1 / ~0.0175 s = 57 req/s), light load again
    rate = lambda t: 90.0 if 4.0 <= t < 9.0 else 20.0
    recs = poisson_queue(rng, 900, rate)
    t_end = recs[-1][0]
    want = M.monitor_run([(t, lr, M.exec_latency(g, c)) for (t, lr, g, c) in recs], W, beta, M.LATENCY, t_end)
    got = run_product(recs, W, beta, B.TS_PLAN_LATENCY, t_end)
    assert len(got) == len(want) > 5
    sw, last = 0, float("nan")
    cur = M.LATENCY
    for (pol, nsw, ratio), (n, wratio, wpol) in zip(got, want):
        if wpol != cur:
            sw, cur = sw + 1, wpol
        if not math.isnan(wratio):
            last = wratio
        assert pol == wpol and nsw == sw, n
        assert (math.isnan(ratio) and math.isnan(last)) or ratio == pytest.approx(last, rel=1e-12), n
    assert {p for (p, _, _) in got} == {M.LATENCY, M.THROUGHPUT}          # the burst is seen and left again


def test_skipping_idle_time_and_late_records():
    h = B.ts_monitor_create(1.0, 1.5, B.TS_PLAN_LATENCY)
    try:
        B.ts_monitor_record(h, 0.5, 4.0, [1.0], 0.0)
        assert B.ts_monitor_advance(h, 0.99)[:3] == (B.TS_PLAN_LATENCY, 0, 0)      # window 0 still open
        pol, closed, sw, ratio = B.ts_monitor_advance(h, 1e6 + 0.5)                  # a long idle stretch
        assert (pol, closed, sw, ratio) == (B.TS_PLAN_THROUGHPUT, 10 ** 6, 1, 4.0)
        with pytest.raises(B.TesseraError):
            B.ts_monitor_record(h, 10.0, 1.0, [1.0], 0.0)                            # its window has closed
        B.ts_monitor_record(h, 1e6 + 0.75, 1.0, [0.5, 0.25], 0.25)
        assert B.ts_monitor_advance(h, 1e6 + 1.0) == (B.TS_PLAN_LATENCY, 10 ** 6 + 1, 2, 1.0)
        with pytest.raises(B.TesseraError):
            B.ts_monitor_record(h, 1e6 + 1.5, 1.0, [], 0.0)                          # no execution time at all
    finally:
        B.ts_monitor_destroy(h)
    for bad in [(0.0, 1.5), (0.3, 0.0), (float("inf"), 1.5)]:
        with pytest.raises(B.TesseraError):
            B.ts_monitor_create(*bad)
