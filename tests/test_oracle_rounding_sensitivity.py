"""What an end-to-end comparison of two bf16 pipelines can and cannot show (oracle only, CPU).

Every kernel boundary of the layer is a bf16 buffer.  A disturbance far below one bf16 ulp in a kernel's result
moves an element of its rounded buffer by a whole ulp with probability disturbance / ulp, so after the rounding
the disturbance has RMS sqrt(disturbance * ulp) instead of `disturbance`: small differences between two
implementations are amplified at every boundary, whatever the implementations are.  The attention kernel keeps
its probabilities in bf16 for the second product (relative error of its result about 2e-3, within its stated
tolerance); this file measures, with the oracle alone, what a disturbance of that size in the attention output
does to the layer output of the boundary-rounding oracle.  The figures explain the end-to-end gate of the
full-size GPU tests: the relative L2 error stays inside the stated 5e-3, the largest element error does not stay
inside 2e-2, and both are properties of the bf16 boundaries, not of a kernel."""
import numpy as np
import pytest
import torch

import workloads as WL
from oracle import decoder_layer as O


_CACHE = {}


def _inputs():
    if not _CACHE:
        shape = WL.CONFIGS["8b_decode"].shape          # full width: H 4096, F 14336 (the error of `out` grows with F)
        wl = WL.Workload("wide", shape, "decode", B=16)
        weights, io, _ = WL.build(wl, seed=4, ctx_lens=[200 + 37 * i for i in range(16)])
        _CACHE["shape"] = shape
        _CACHE["w"] = {k: WL.as_f64(v) for k, v in weights.items()}
        _CACHE["io"] = {k: WL.as_f64(v) for k, v in io.items()}
    return _CACHE["shape"], _CACHE["w"], {k: v.copy() for k, v in _CACHE["io"].items()}


def _layer(perturb=None, rounded=True):
    shape, w64, io64 = _inputs()
    return O.layer_forward(shape, w64, io64, "decode", round_boundaries=rounded, perturb=perturb)


def _noise(rel, seed=0):
    rng = np.random.default_rng(seed)
    return lambda a: a * (1.0 + rel * rng.standard_normal(a.shape))


def _rel(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(a))


def test_no_perturbation_changes_nothing():
    a, b = _layer(), _layer(perturb={})
    for n in O.BOUNDARY_ORDER_DENSE:
        assert np.array_equal(a[n], b[n])
    # without rounding a disturbance passes through at its own size
    e, p = _layer(rounded=False), _layer(perturb={"attn": _noise(2e-3)}, rounded=False)
    assert _rel(e["attn"], p["attn"]) == pytest.approx(2e-3, rel=0.1)
    _CACHE["unrounded_out"] = _rel(e["out"], p["out"])
    assert _CACHE["unrounded_out"] < 6e-4       # the attention branch is a small part of the residual stream


def test_attention_sized_disturbance_through_the_bf16_boundaries():
    a = _layer()
    p = _layer(perturb={"attn": _noise(2e-3)})
    differing = {n: float(np.mean(a[n] != p[n])) for n in O.BOUNDARY_ORDER_DENSE}
    rel = {n: _rel(a[n], p[n]) for n in O.BOUNDARY_ORDER_DENSE}
    print({n: (round(differing[n], 3), f"{rel[n]:.2e}", round(float(np.abs(a[n] - p[n]).max()), 4)) for n in rel})
    assert differing["h1"] == 0.0 and differing["qkv"] == 0.0
    # a good part of the attention outputs round to another bf16 value, and although nothing but roundings
    # happens to the disturbance afterwards, about half of the layer outputs end up on another bf16 value
    assert 0.15 < differing["attn"] < 0.6
    assert differing["x2"] < differing["gate_up"] < differing["act"]
    assert differing["out"] > 0.3
    # relative L2 of the output: several times what the un-rounded pipeline shows (test above), and still inside
    # the stated 5e-3
    assert 2e-3 < rel["out"] < 5e-3
    assert rel["out"] > 4 * _CACHE.get("unrounded_out", 4e-4)
    # the largest element error is a few bf16 ulps of an O(1) value: above the stated 2e-2
    assert np.abs(a["out"] - p["out"]).max() > 2e-2
    assert np.abs(a["act"] - p["act"]).max() > 2e-2


def test_a_disturbance_far_below_one_ulp_is_amplified():
    """A relative disturbance of 1e-5 in the attention output (a thousandth of a bf16 ulp) leaves a relative L2
    error of the layer output some hundred times its own size."""
    a = _layer()
    small = _rel(a["out"], _layer(perturb={"attn": _noise(1e-5, 1)})["out"])
    assert small > 5e-4
