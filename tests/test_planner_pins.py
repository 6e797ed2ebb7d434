"""Pins for the dependency-graph and policy-planner oracle (CPU only).

Hand-worked graphs and placements, closed forms, and an independent library
routine (scipy max-flow) for the two-GPU latency objective.  Nothing here calls
the C++ implementation.
"""
import itertools

import numpy as np
import pytest

from oracle import planner as P

INF = float("inf")


def K(reads=(), writes=()):
    return {"reads": [tuple(r) for r in reads], "writes": [tuple(w) for w in writes]}


def full(addr, n):
    return (addr, n, n)


# ------------------------------------------------------------------ dependency graph
def test_ddg_chain_with_skip_connection():
    # k0 writes A; k1 reads A writes B; k2 reads B writes C; k3 reads C and A (skip) writes D
    A, B, C, D = 0, 1000, 2000, 3000
    ks = [K(writes=[full(A, 100)]), K([full(A, 100)], [full(B, 50)]), K([full(B, 50)], [full(C, 70)]),
          K([full(C, 70), full(A, 100)], [full(D, 10)])]
    edges, cross = P.ddg_build(ks)
    assert edges == {(0, 1): 100, (1, 2): 50, (2, 3): 70, (0, 3): 100}
    assert cross == {}


def test_ddg_only_true_dependencies_and_most_recent_writer():
    # write-after-read and write-after-write create no edge; a read sees the LAST writer only
    A = 0
    ks = [K(writes=[full(A, 64)]), K(reads=[full(A, 64)]), K(writes=[full(A, 64)]), K(reads=[full(A, 64)])]
    edges, cross = P.ddg_build(ks)
    assert edges == {(0, 1): 64, (2, 3): 64}
    # k1 of the next iteration reads what k0 of that iteration wrote, never k2 of the previous one
    assert cross == {}


def test_ddg_partial_overlap_is_split_between_writers():
    # bytes [0,100) by k0, then k1 overwrites [40,60); k2 reads [30,80)
    ks = [K(writes=[full(0, 100)]), K(writes=[full(40, 20)]), K(reads=[full(30, 50)])]
    edges, _ = P.ddg_build(ks)
    assert edges == {(1, 2): 20, (0, 2): 30}          # 10 + 20 bytes of k0 survive around k1's 20


def test_ddg_in_place_kernel_has_no_self_edge():
    # k1 rotates a buffer in place (reads and writes it): it depends on k0, k2 depends on k1 only
    ks = [K(writes=[full(0, 32)]), K([full(0, 32)], [full(0, 32)]), K(reads=[full(0, 32)])]
    edges, cross = P.ddg_build(ks)
    assert edges == {(0, 1): 32, (1, 2): 32}
    assert cross == {}


def test_ddg_unwritten_input_and_weights_give_no_edge():
    ks = [K(reads=[full(0, 10), full(500, 99)], writes=[full(100, 10)]), K(reads=[full(100, 10), full(500, 99)])]
    edges, cross = P.ddg_build(ks)
    assert edges == {(0, 1): 10} and cross == {}


def test_ddg_cross_iteration_cache():
    # a cache of 1000 bytes: k0 appends 8 bytes somewhere inside it (hull = whole cache), k1 reads all of
    # it.  Inside an iteration the 8 appended bytes flow k0 -> k1; nothing else writes the cache, so the
    # previous iteration's append is NOT visible as a separate dependency (same writer kernel, same hull).
    ks = [K(writes=[(0, 1000, 8)]), K(reads=[(0, 1000, 1000)])]
    edges, cross = P.ddg_build(ks)
    assert edges == {(0, 1): 8} and cross == {}
    # a buffer read early in the iteration and written late: the value comes from the previous iteration
    ks = [K(reads=[full(0, 16)], writes=[full(100, 4)]), K(reads=[full(100, 4)], writes=[full(0, 16)])]
    edges, cross = P.ddg_build(ks)
    assert edges == {(0, 1): 4}
    assert cross == {(1, 0): 16}


def test_ddg_append_position_advances_between_iterations():
    # two cache rows of 10 slots x 4 bytes; k0 appends one slot per row (slot 3 now, slot 4 next iteration),
    # k1 reads both rows whole.  Inside the iteration 2 x 4 new bytes flow; the slots appended by the previous
    # iteration are still the latest content of their bytes, so 2 x 4 bytes arrive across the iteration boundary.
    rows = [0, 40]
    ks = [K(writes=[(r + 3 * 4, 4, 4, 4) for r in rows]), K(reads=[(0, 80, 80)])]
    edges, cross = P.ddg_build(ks)
    assert edges == {(0, 1): 8}
    assert cross == {(0, 1): 8}
    # without the advance the second iteration overwrites the same slots: nothing crosses
    ks = [K(writes=[(r + 3 * 4, 4, 4) for r in rows]), K(reads=[(0, 80, 80)])]
    assert P.ddg_build(ks) == ({(0, 1): 8}, {})


def test_ddg_flow_is_bounded_by_both_sides():
    rng = np.random.default_rng(5)
    for _ in range(50):
        n = int(rng.integers(2, 7))
        ks = []
        for _k in range(n):
            acc = lambda: [(int(rng.integers(0, 40)), int(e), int(rng.integers(1, e + 1)))
                           for e in rng.integers(1, 30, size=int(rng.integers(0, 3)))]
            ks.append({"reads": acc(), "writes": acc()})
        edges, cross = P.ddg_build(ks)
        for (i, j), d in edges.items():
            assert i < j and d > 0                                   # execution order is preserved
            assert d <= sum(b for (_, _, b) in ks[j]["reads"]) * max(1, len(ks[i]["writes"]))
        for (i, j), d in cross.items():
            assert i >= j and d > 0                                  # only a later (or the same) kernel can feed the next iteration


# ------------------------------------------------------------------ objectives, by hand
def test_two_kernels_one_edge_all_four_placements():
    t = [[1.0, 3.0], [4.0, 2.0]]
    edges = {(0, 1): 100.0}
    bw = [[INF, 50.0], [25.0, INF]]
    lat = [[0.0, 0.5], [0.25, 0.0]]
    # c^{0,1} = 0.5 + 100/50 = 2.5 ; c^{1,0} = 0.25 + 100/25 = 4.25
    want_lat = {(0, 0): 5.0, (1, 1): 5.0, (0, 1): 1.0 + 2.0 + 2.5, (1, 0): 3.0 + 4.0 + 4.25}
    want_thr = {(0, 0): 5.0, (1, 1): 5.0, (0, 1): max(1.0, 0.0, 2.0, 2.5), (1, 0): max(4.0, 4.25, 3.0, 0.0)}
    for pl in itertools.product(range(2), repeat=2):
        assert P.policy_objective(pl, t, edges, bw, lat, 2, "latency") == pytest.approx(want_lat[pl])
        assert P.policy_objective(pl, t, edges, bw, lat, 2, "throughput") == pytest.approx(want_thr[pl])
    assert P.plan_bruteforce(t, edges, bw, lat, "throughput")[0] == pytest.approx(2.5)
    assert P.plan_bruteforce(t, edges, bw, lat, "latency")[0] == pytest.approx(5.0)


def test_incoming_edges_only_count_on_the_receiver():
    # three kernels on a line, the middle one on the other GPU: GPU 1 receives one edge, GPU 0 receives one
    t = [[1, 1], [1, 1], [1, 1]]
    edges = {(0, 1): 10.0, (1, 2): 30.0}
    bw = [[INF, 10.0], [10.0, INF]]
    lat = [[0, 0], [0, 0]]
    T, M = P.policy_terms((0, 1, 0), t, edges, bw, lat, 2)
    assert T == [2.0, 1.0] and M == [3.0, 1.0]


def test_free_communication_closed_forms():
    rng = np.random.default_rng(7)
    t = rng.uniform(1, 5, size=(7, 2)).tolist()
    edges = {(i, i + 1): 10.0 for i in range(6)}
    bw = [[INF, INF], [INF, INF]]
    lat = [[0, 0], [0, 0]]
    best, place = P.plan_bruteforce(t, edges, bw, lat, "latency")
    assert best == pytest.approx(sum(min(r) for r in t))            # every kernel on its faster GPU
    assert place == [int(np.argmin(r)) for r in t]
    # identical GPUs, free communication: throughput objective = balanced two-way partition
    t = [[3, 3], [3, 3], [2, 2], [2, 2], [2, 2]]
    best, _ = P.plan_bruteforce(t, {}, bw, lat, "throughput")
    assert best == 6.0


def test_prohibitive_communication_and_single_gpu():
    t = [[2.0, 1.0], [2.0, 1.5], [1.0, 3.0]]
    edges = {(0, 1): 1.0, (1, 2): 1.0, (0, 2): 1.0}
    bw = [[INF, 1e-9], [1e-9, INF]]
    lat = [[0, 0], [0, 0]]
    for obj in ("latency", "throughput"):
        best, place = P.plan_bruteforce(t, edges, bw, lat, obj)
        assert len(set(place)) == 1 and best == pytest.approx(5.0)  # GPU 0: 5.0, GPU 1: 5.5
    best, place = P.plan_bruteforce([[r[0]] for r in t], edges, [[INF]], [[0]], "throughput")
    assert best == pytest.approx(5.0) and place == [0, 0, 0]


def test_two_gpu_latency_objective_is_a_minimum_cut():
    """With two GPUs the latency objective is a two-label energy with non-negative cut costs: its
    minimum equals an s-t minimum cut, computed here by scipy's max-flow on integer data."""
    maximum_flow = pytest.importorskip("scipy.sparse.csgraph").maximum_flow
    from scipy.sparse import csr_matrix
    rng = np.random.default_rng(11)
    for _ in range(20):
        n = int(rng.integers(3, 9))
        t = rng.integers(1, 20, size=(n, 2)).astype(float).tolist()
        pairs = [(i, j) for i in range(n) for j in range(i + 1, n) if rng.random() < 0.4]
        d = {p: float(rng.integers(1, 10)) for p in pairs}
        bw = [[INF, 1.0], [1.0, INF]]                  # c = d both ways
        lat = [[0, 0], [0, 0]]
        best, _ = P.plan_bruteforce(t, d, bw, lat, "latency")
        # s = node n (label 0 side), tt = node n+1.  Kernel k on GPU 1 (cut s->k) pays t[k][1];
        # on GPU 0 (cut k->t) pays t[k][0]; an edge pays d when its ends differ.
        cap = np.zeros((n + 2, n + 2), dtype=np.int32)
        for k in range(n):
            cap[n, k] = int(t[k][1])
            cap[k, n + 1] = int(t[k][0])
        for (i, j), v in d.items():
            cap[i, j] += int(v)
            cap[j, i] += int(v)
        flow = maximum_flow(csr_matrix(cap), n, n + 1).flow_value
        assert best == pytest.approx(float(flow))


@pytest.mark.parametrize("objective", ["throughput", "latency"])
def test_milp_formulation_attains_the_bruteforce_optimum(objective):
    """The mixed-integer programme of Sec. 3.2 (binary placements, linearised edge products, W above every T_g
    and M_g) handed to a solver gives what enumeration gives: pins `plan_milp`, the reference at sizes that
    cannot be enumerated."""
    import numpy as np
    rng = np.random.default_rng(5)
    for trial in range(6):
        nk, ng = 6 + trial % 3, 2 + trial % 2
        t = [[float(rng.uniform(1, 10)) for _ in range(ng)] for _ in range(nk)]
        edges = {(i, j): float(rng.uniform(1, 50)) for i in range(nk) for j in range(i + 1, nk) if rng.random() < 0.35}
        bw = [[float("inf") if a == b else float(rng.uniform(5, 20)) for b in range(ng)] for a in range(ng)]
        lat = [[0.0 if a == b else float(rng.uniform(0, 1)) for b in range(ng)] for a in range(ng)]
        best, _ = P.plan_bruteforce(t, edges, bw, lat, objective)
        value, place, bound = P.plan_milp(t, edges, bw, lat, objective)
        assert value == pytest.approx(best, rel=1e-9)
        assert bound <= value * (1 + 1e-9) and bound >= best * (1 - 1e-6)
        assert P.policy_objective(place, t, edges, bw, lat, ng, objective) == pytest.approx(value)
    # times of a few microseconds (below the solver's absolute tolerances unless the programme is rescaled)
    t = [[3e-6, 9e-6], [5e-6, 6e-6], [4e-6, 4e-6], [7e-6, 30e-6], [2e-6, 2.5e-6]]
    edges = {(0, 1): 1e5, (1, 2): 2e5, (2, 3): 1e5, (0, 4): 5e4}
    bw = [[float("inf"), 25e9], [25e9, float("inf")]]
    lat = [[0.0, 1e-7], [1e-7, 0.0]]
    best, _ = P.plan_bruteforce(t, edges, bw, lat, objective)
    assert P.plan_milp(t, edges, bw, lat, objective)[0] == pytest.approx(best, rel=1e-9)
