"""CPU oracle for the online monitor's policy switching (TEST INFRASTRUCTURE, not product).

Only tests/ may import this.  It shares no code with the C++ implementation in
paper_2604_10180_amd/csrc/monitor.hip and never imports it.

What it is: the queueing-aware switch of Sec. 3.4 written as the definition.  Time is cut into fixed
windows of length W.  At each window boundary the mean request latency L_req and the mean pure
execution latency L_exec (kernel-group compute time plus communication time, queueing excluded) of
the requests that finished inside the window are formed; their ratio L_req / L_exec measures
queueing pressure; a ratio above the threshold beta selects the throughput-oriented policy, a ratio
at or below it the latency-oriented one.  Defaults of Sec. 5.4: W = 0.3 s, beta = 1.5.

Readings taken (the paper leaves them open):
  M1  a request belongs to the window in which it completes; window n is [n W, (n+1) W).
  M2  the indicator is the ratio of the two window means, not the mean of per-request ratios.
  M3  a window without completions carries no information: the policy stays.
  M4  "high" means strictly above beta.
  M5  L_exec of a request = sum of its kernel-group latencies + its communication time.

Pins (tests/test_monitor_pins.py): a hand-worked trace, a deterministic single-server queue with
closed-form waiting times, limits of beta, invariance under a change of time unit.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

LATENCY, THROUGHPUT = 1, 0          # same numbering as the planner's objectives


def exec_latency(group_latencies: Sequence[float], comm: float) -> float:
    """M5: compute time of all kernel groups plus communication time."""
    return sum(group_latencies) + comm


def monitor_run(requests: Sequence[Tuple[float, float, float]], W: float = 0.3, beta: float = 1.5,
                initial_policy: int = LATENCY, t_end: float | None = None) -> List[Tuple[int, float, int]]:
    """requests: (completion time, request latency, execution latency), any order.

    Returns one entry per window that closed by t_end (default: the last completion):
    (window index, ratio or nan for an empty window, policy in effect AFTER the boundary)."""
    if not requests and t_end is None:
        return []
    last = max(r[0] for r in requests) if requests else 0.0
    horizon = last if t_end is None else t_end
    n_windows = int(math.floor(horizon / W))           # windows [nW, (n+1)W) with (n+1)W <= horizon
    policy = initial_policy
    out = []
    for n in range(n_windows):
        inside = [r for r in requests if n * W <= r[0] < (n + 1) * W]
        if not inside:
            out.append((n, float("nan"), policy))
            continue
        l_req = sum(r[1] for r in inside) / len(inside)
        l_exec = sum(r[2] for r in inside) / len(inside)
        ratio = l_req / l_exec
        policy = THROUGHPUT if ratio > beta else LATENCY
        out.append((n, ratio, policy))
    return out


def switch_count(decisions: Sequence[Tuple[int, float, int]], initial_policy: int = LATENCY) -> int:
    n, cur = 0, initial_policy
    for (_, _, p) in decisions:
        if p != cur:
            n += 1
            cur = p
    return n
