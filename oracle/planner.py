"""CPU oracle for the kernel analyzer's dependency graph and the policy planner
(TEST INFRASTRUCTURE, not product).

Only tests/ may import this.  It shares no code with the C++ implementation in
paper_2604_10180_amd/csrc/planner.hip and never imports it.

What it is:

* `ddg_build` -- the data-dependency graph of Sec. 3.1 ("Data dependency
  analysis"), written as the definition: kernels are visited in execution
  order, a read depends on the MOST RECENT earlier writer of the bytes it
  reads (true, read-after-write dependencies only), a kernel never depends on
  itself, one edge per (writer, reader) pair annotated with the bytes that
  flow.  Cross-iteration dependencies are found the way the paper describes:
  the kernel list is run for two iterations and a read in the second iteration
  whose most recent writer ran in the first is flagged.
* `plan_milp` -- the same two objectives as the mixed-integer linear programme the paper
  hands to its solver (Sec. 3.2): binary x[k,g], one GPU per kernel, the product
  y = x[i,u] x[j,g] of every edge replaced by a continuous y with y >= x[i,u] + x[j,g] - 1
  (the standard linearisation; costs are non-negative and minimised, so the lower bound on y
  is the only one that binds), T_g and M_g below a common W, minimise W (throughput), or
  minimise sum t x + sum c y (latency).  scipy's MILP routine (HiGHS) serves as the solver,
  a library step as the commercial solver is in the paper.  Used to check the product planner at
  sizes where enumeration is impossible.
* `policy_objective` / `plan_bruteforce` -- the two objectives of Sec. 3.2
  evaluated literally from their formulas (placement variables x, computation
  time T_g, communication time M_g with c = l + d / bw on cut edges, stage
  time W_g = max(T_g, M_g); throughput objective min max_g W_g, latency
  objective min sum t x + sum of c over cut edges) and minimised by
  enumerating every placement.  Exponential on purpose.

Readings taken (the paper leaves them open):
  P1  an access is a byte range [addr, addr + extent) plus the number of bytes
      actually touched inside it (`bytes <= extent`; the analyzer of Sec. 3.1
      keeps a [min, max] hull per instruction).  The bytes that flow along a
      dependency are min(overlap of the two ranges, bytes written, bytes read).
  P2  several buffers between the same two kernels add up into one edge.
  P3  all reads of a kernel happen before its writes.
  P4  cross-iteration edges are reported separately and carry no cost in the
      objectives (the method replicates such buffers and ships deltas in the
      background, Sec. 4).
  P5  M_g counts incoming cut edges only, as printed; the latency objective
      counts every cut edge once.
  P6  the two profiled iterations of Sec. 3.1 are consecutive real iterations:
      an append-style access (the KV cache row of the token being decoded)
      lands one position further in the second iteration.  An access may carry
      a fourth element, the bytes its range advances per iteration (default 0).

Pins (tests/test_planner_pins.py): `plan_milp` against `plan_bruteforce` on random
problems; hand-worked graphs and placements, closed
forms (free communication, prohibitive communication, one GPU, balanced
partition), and for two GPUs the latency objective against a max-flow/min-cut
computed by scipy (the objective is a submodular two-label energy).
No function here is "parity unpinned".
"""
from __future__ import annotations

import itertools
from typing import Dict, List, Sequence, Tuple

Access = Tuple[int, ...]               # (addr, extent, bytes touched[, advance per iteration])


def _at(access, it: int):
    """The access as it happens in iteration `it` (reading P6)."""
    addr, extent, nbytes = access[:3]
    step = access[3] if len(access) > 3 else 0
    return addr + it * step, extent, nbytes


def _subtract(intervals: List[Tuple[int, int]], lo: int, hi: int) -> List[Tuple[int, int]]:
    """Remove [lo, hi) from a list of disjoint half-open intervals."""
    out = []
    for a, b in intervals:
        if hi <= a or b <= lo:
            out.append((a, b))
            continue
        if a < lo:
            out.append((a, lo))
        if hi < b:
            out.append((hi, b))
    return out


def ddg_build(kernels: Sequence[dict]):
    """kernels[k] = {"reads": [Access...], "writes": [Access...]} in execution order.

    Returns (edges, cross) where both are dicts {(writer, reader): bytes}; `edges` holds the
    dependencies inside one iteration, `cross` those from the previous iteration.
    """
    n = len(kernels)
    log: List[Tuple[int, int, int, int, int]] = []      # (iteration, kernel, addr, extent, bytes) of every write so far
    edges: Dict[Tuple[int, int], int] = {}
    cross: Dict[Tuple[int, int], int] = {}
    for it in range(2):
        for k in range(n):
            for access in kernels[k]["reads"]:
                addr, extent, nbytes = _at(access, it)
                uncovered = [(addr, addr + extent)]
                for (wit, wk, waddr, wext, wbytes) in reversed(log):   # most recent writer first
                    if not uncovered:
                        break
                    ov = 0
                    for a, b in uncovered:
                        ov += max(0, min(b, waddr + wext) - max(a, waddr))
                    if ov == 0:
                        continue
                    uncovered = _subtract(uncovered, waddr, waddr + wext)
                    if wit == it and wk == k:
                        continue                                        # a kernel does not depend on itself
                    flow = min(ov, wbytes, nbytes)
                    if it == 1:
                        target = edges if wit == 1 else cross
                        target[(wk, k)] = target.get((wk, k), 0) + flow
            for access in kernels[k]["writes"]:
                addr, extent, nbytes = _at(access, it)
                log.append((it, k, addr, extent, nbytes))
    return edges, cross


def transfer_cost(d: float, u: int, g: int, bw, lat) -> float:
    """c_ij^{u,g} = l_{u,g} + d_ij / bw_{u,g}."""
    return lat[u][g] + d / bw[u][g]


def policy_terms(place: Sequence[int], t, edges: Dict[Tuple[int, int], float], bw, lat, n_gpus: int):
    """(T_g, M_g) of a placement: computation and incoming-communication time per GPU."""
    T = [0.0] * n_gpus
    M = [0.0] * n_gpus
    for k, g in enumerate(place):
        T[g] += t[k][g]
    for (i, j), d in edges.items():
        u, g = place[i], place[j]
        if u != g:
            M[g] += transfer_cost(d, u, g, bw, lat)
    return T, M


def policy_objective(place, t, edges, bw, lat, n_gpus: int, objective: str) -> float:
    T, M = policy_terms(place, t, edges, bw, lat, n_gpus)
    if objective == "throughput":
        return max(max(T[g], M[g]) for g in range(n_gpus))
    if objective == "latency":
        return sum(T) + sum(M)
    raise ValueError(objective)


def plan_bruteforce(t, edges, bw, lat, objective: str):
    """Enumerate every placement; returns (best objective value, one best placement)."""
    n_k, n_g = len(t), len(t[0])
    best, best_place = None, None
    for place in itertools.product(range(n_g), repeat=n_k):
        v = policy_objective(place, t, edges, bw, lat, n_g, objective)
        if best is None or v < best:
            best, best_place = v, place
    return best, list(best_place)


def plan_milp(t, edges: Dict[Tuple[int, int], float], bw, lat, objective: str, rel_gap: float = 1e-9,
              time_limit: float = 120.0):
    """The MILP of Sec. 3.2 solved by scipy.optimize.milp.

    Returns (objective value of the placement found, placement, dual bound): the dual bound is the
    solver's proven lower bound of the optimum (equal to the value up to rel_gap when it finishes).
    """
    import numpy as np
    from scipy.optimize import Bounds, LinearConstraint, milp
    from scipy.sparse import lil_matrix

    n_k, n_g = len(t), len(t[0])
    pairs = [(u, g) for u in range(n_g) for g in range(n_g) if u != g]
    elist = list(edges.items())
    # The solver works with absolute tolerances (about 1e-6 on the objective), so the programme is stated in
    # units in which a kernel takes about 100: times in seconds of a few microseconds would be below them.
    unit = 100.0 / max(1e-300, float(np.mean([max(row) for row in t])))
    nx = n_k * n_g
    ny = len(elist) * len(pairs)
    n = nx + ny + 1                       # ... + W
    X = lambda k, g: k * n_g + g
    Y = lambda e, p: nx + e * len(pairs) + p
    Wv = n - 1
    cost = np.zeros(ny)
    for e, ((i, j), d) in enumerate(elist):
        for p, (u, g) in enumerate(pairs):
            cost[e * len(pairs) + p] = transfer_cost(d, u, g, bw, lat) * unit
    rows, lo, hi = [], [], []
    A = lil_matrix((n_k + ny + 2 * n_g, n))
    r = 0
    for k in range(n_k):                  # one GPU per kernel
        for g in range(n_g):
            A[r, X(k, g)] = 1.0
        lo.append(1.0); hi.append(1.0); r += 1
    for e, ((i, j), d) in enumerate(elist):   # y >= x_iu + x_jg - 1
        for p, (u, g) in enumerate(pairs):
            A[r, X(i, u)] = 1.0
            A[r, X(j, g)] = 1.0
            A[r, Y(e, p)] = -1.0
            lo.append(-np.inf); hi.append(1.0); r += 1
    c = np.zeros(n)
    if objective == "throughput":
        for g in range(n_g):              # T_g <= W
            for k in range(n_k):
                A[r, X(k, g)] = t[k][g] * unit
            A[r, Wv] = -1.0
            lo.append(-np.inf); hi.append(0.0); r += 1
        for g in range(n_g):              # M_g <= W
            for e in range(len(elist)):
                for p, (u, gg) in enumerate(pairs):
                    if gg == g:
                        A[r, Y(e, p)] = cost[e * len(pairs) + p]
            A[r, Wv] = -1.0
            lo.append(-np.inf); hi.append(0.0); r += 1
        c[Wv] = 1.0
    elif objective == "latency":
        for k in range(n_k):
            for g in range(n_g):
                c[X(k, g)] = t[k][g] * unit
        c[nx:nx + ny] = cost
    else:
        raise ValueError(objective)
    A = A[:r].tocsr()
    integrality = np.zeros(n)
    integrality[:nx] = 1
    ub = np.ones(n)
    ub[Wv] = np.inf
    res = milp(c, constraints=LinearConstraint(A, np.array(lo), np.array(hi)), integrality=integrality,
               bounds=Bounds(np.zeros(n), ub), options={"mip_rel_gap": rel_gap, "time_limit": time_limit})
    if res.x is None:
        raise RuntimeError(f"MILP not solved: {res.message}")
    place = [int(np.argmax(res.x[k * n_g:(k + 1) * n_g])) for k in range(n_k)]
    value = policy_objective(place, t, edges, bw, lat, n_g, objective)
    bound = getattr(res, "mip_dual_bound", None)
    return value, place, (float(bound) if bound is not None else float(res.fun)) / unit
