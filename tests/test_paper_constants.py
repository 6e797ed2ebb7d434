"""The constants taken over from the paper (tests/golden/paper_constants.txt) are consistent with what the
paper says about them elsewhere, and the code uses exactly these values (CPU only)."""
import inspect
import os

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def records():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_constants.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        kind, name, *kv = line.split()
        out[(kind, name)] = {kv[i]: float(kv[i + 1]) for i in range(0, len(kv), 2)}
    return out


def test_table_matches_the_ratios_quoted_in_the_text():
    r = records()
    a, l = r[("gpu", "A100")], r[("gpu", "L40s")]
    q = r[("ratio", "L40s_over_A100")]
    assert round(l["cuda_tflops"] / a["cuda_tflops"], 1) == q["cuda"]
    assert round(l["tensor_tflops"] / a["tensor_tflops"], 1) == q["tensor"]
    assert round(l["bw_gbs"] / a["bw_gbs"], 2) == q["bandwidth"]
    assert l["price"] == 1.0                                   # prices are normalised by the L40s
    assert len([k for k in r if k[0] == "gpu"]) == 5


def test_planner_demonstration_uses_the_table_and_the_testbed_link():
    import bench
    r = records()
    assert bench.MODELLED_GPUS["L40S-like"] == (r[("gpu", "L40s")]["tensor_tflops"], r[("gpu", "L40s")]["bw_gbs"])
    assert bench.MODELLED_GPUS["H100-like"] == (r[("gpu", "H100")]["tensor_tflops"], r[("gpu", "H100")]["bw_gbs"])
    link = inspect.signature(bench.plan_section).parameters["link_GBps"].default
    assert link == r[("link", "testbed")]["gbps"] / 8.0          # 200 Gbit/s = 25 GB/s


def test_monitor_defaults_are_the_papers():
    from paper_2604_10180_amd import binding as B
    r = records()[("monitor", "default")]
    sig = inspect.signature(B.ts_monitor_create).parameters
    assert sig["window_s"].default == r["window_s"] and sig["beta"].default == r["beta"]
    assert sig["initial_policy"].default == B.TS_PLAN_LATENCY


def test_monitor_host_cases_cover_the_named_settings():
    import test_monitor_host as T
    r = records()
    cases = None
    for mark in T.test_decisions_match_the_oracle_on_bursty_poisson_load.pytestmark:
        if mark.name == "parametrize":
            cases = set(mark.args[1])
    for name in ("default", "aggressive", "conservative"):
        assert (r[("monitor", name)]["window_s"], r[("monitor", name)]["beta"]) in cases
