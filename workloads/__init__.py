"""Seeded synthetic workloads for the decoder-layer hot path.

This module only *draws numbers and names shapes*.  It holds none of the
method's arithmetic: no normalisation, no matmul, no softmax, no rotary angle.
It is the one module that both the CPU oracle's tests and the HIP path's
tests/benchmarks import, so that the two sides see bit-identical inputs.

Recipe (every tensor is drawn in fp32 from a `torch.Generator` seeded by the
caller, rounded ONCE to bf16 with round-to-nearest-even, and handed out as a
bf16 tensor; `as_f64` widens the same values for the oracle):

  * weights                     N(0, 0.02)
  * RMSNorm gains               1 + 0.02 * N(0, 1)
  * activations x, cached K, V  N(0, 1)
  * router matrix               N(0, 0.02)
  * ragged context lengths      integers uniform in [lo, hi]

Draw order is part of the contract and is fixed by the code below:
lengths (if ragged) -> weights (gamma1, w_qkv, w_o, gamma2, [w_router],
w_gate_up, w_down) -> x -> per sequence: K rows then V rows.

The five named workloads mirror the five benchmark configurations (tiny layer,
8B-shaped decode, 8B-shaped prefill, 8-expert top-2 MoE decode, 70B-shaped
ragged decode run as four micro-batches).  They stand in for the model shapes
and context lengths of the paper's serving experiments (Sec. 5.1), whose
weights and request traces are not available; only shapes and rough context
lengths carry over.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch


@dataclass(frozen=True)
class LayerShape:
    H: int            # hidden size
    nq: int           # query heads
    nkv: int          # key/value heads (nq % nkv == 0)
    d: int            # head dimension
    F: int            # SwiGLU inner width (per expert for MoE)
    E: int = 0        # number of experts, 0 = dense MLP
    k: int = 0        # experts per token
    eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def n_qkv(self) -> int:
        return (self.nq + 2 * self.nkv) * self.d


@dataclass(frozen=True)
class Workload:
    name: str
    shape: LayerShape
    mode: str                      # "decode" | "prefill"
    B: int                         # sequences in the call
    ctx: int = 0                   # decode: cached positions per sequence (equal lengths)
    ctx_range: Optional[tuple] = None   # decode: (lo, hi) inclusive, ragged lengths
    seq_tokens: int = 0            # prefill: tokens per sequence
    n_micro: int = 1               # micro-batches for the pipeline step
    seed: int = 0

    @property
    def T(self) -> int:
        return self.B if self.mode == "decode" else self.B * self.seq_tokens


_L8B = LayerShape(H=4096, nq=32, nkv=8, d=128, F=14336)

CONFIGS: Dict[str, Workload] = {
    "tiny": Workload("tiny", LayerShape(H=256, nq=4, nkv=2, d=64, F=688), "decode", B=2, ctx=128),
    "8b_decode": Workload("8b_decode", _L8B, "decode", B=64, ctx=2048),
    "8b_prefill": Workload("8b_prefill", _L8B, "prefill", B=4, seq_tokens=2048),
    "moe_decode": Workload("moe_decode", replace(_L8B, E=8, k=2), "decode", B=256, ctx=1024),
    "70b_pipeline": Workload("70b_pipeline", LayerShape(H=8192, nq=64, nkv=8, d=128, F=28672),
                             "decode", B=32, ctx_range=(512, 32768), n_micro=4),
}


def _bf16(t: torch.Tensor) -> torch.Tensor:
    return t.to(torch.bfloat16)


def _randn(gen: torch.Generator, *shape, std: float = 1.0, mean: float = 0.0) -> torch.Tensor:
    t = torch.randn(*shape, generator=gen, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    if mean != 0.0:
        t.add_(mean)
    return _bf16(t)


def as_f64(t: torch.Tensor) -> np.ndarray:
    """Widen a (bf16/fp32/int) CPU tensor to a float64 / int64 numpy array (exact)."""
    if t.dtype in (torch.int32, torch.int64):
        return t.cpu().numpy().astype(np.int64)
    return t.detach().cpu().to(torch.float64).numpy()


def as_f32(t: torch.Tensor) -> np.ndarray:
    """Widen a bf16 CPU tensor to float32 numpy (exact; used for very large caches)."""
    return t.detach().cpu().to(torch.float32).numpy()


def make_weights(shape: LayerShape, gen: torch.Generator) -> Dict[str, torch.Tensor]:
    s = shape
    w: Dict[str, torch.Tensor] = {}
    w["gamma1"] = _randn(gen, s.H, std=0.02, mean=1.0)
    w["w_qkv"] = _randn(gen, s.n_qkv, s.H, std=0.02)
    w["w_o"] = _randn(gen, s.H, s.nq * s.d, std=0.02)
    w["gamma2"] = _randn(gen, s.H, std=0.02, mean=1.0)
    if s.E > 0:
        w["w_router"] = _randn(gen, s.E, s.H, std=0.02)
        w["w_gate_up"] = torch.stack([_randn(gen, 2 * s.F, s.H, std=0.02) for _ in range(s.E)])
        w["w_down"] = torch.stack([_randn(gen, s.H, s.F, std=0.02) for _ in range(s.E)])
    else:
        w["w_gate_up"] = _randn(gen, 2 * s.F, s.H, std=0.02)
        w["w_down"] = _randn(gen, s.H, s.F, std=0.02)
    return w


def make_decode_io(shape: LayerShape, ctx_lens: Sequence[int], gen: torch.Generator,
                   Lcap: Optional[int] = None, tail_fill: float = 0.0) -> Dict[str, torch.Tensor]:
    """One new token per sequence; sequence b has ctx_lens[b] cached positions.

    The new token sits at position ctx_lens[b] and is appended there, so
    Lcap >= max(ctx_lens) + 1.  Cache slots at and beyond ctx_lens[b] are
    filled with `tail_fill` (tests pass NaN to prove nothing there is read).
    """
    s = shape
    B = len(ctx_lens)
    if Lcap is None:
        Lcap = int(max(ctx_lens)) + 1
    assert Lcap >= int(max(ctx_lens)) + 1
    io: Dict[str, torch.Tensor] = {}
    io["x"] = _randn(gen, B, s.H)
    kc = torch.full((B, s.nkv, Lcap, s.d), tail_fill, dtype=torch.bfloat16)
    vc = torch.full((B, s.nkv, Lcap, s.d), tail_fill, dtype=torch.bfloat16)
    for b, L in enumerate(ctx_lens):
        L = int(L)
        if L > 0:
            kc[b, :, :L] = _randn(gen, s.nkv, L, s.d)
            vc[b, :, :L] = _randn(gen, s.nkv, L, s.d)
    io["kcache"], io["vcache"] = kc, vc
    io["pos"] = torch.tensor([int(L) for L in ctx_lens], dtype=torch.int32)
    io["seq_id"] = torch.arange(B, dtype=torch.int32)
    io["seq_lens"] = io["pos"] + 1          # keys attended after the append
    return io


def make_prefill_io(shape: LayerShape, seq_tokens: Sequence[int], gen: torch.Generator,
                    Lcap: Optional[int] = None, tail_fill: float = 0.0) -> Dict[str, torch.Tensor]:
    """Fresh sequences: sequence b has seq_tokens[b] prompt tokens at positions 0..n-1."""
    s = shape
    B = len(seq_tokens)
    T = int(sum(seq_tokens))
    if Lcap is None:
        Lcap = int(max(seq_tokens))
    io: Dict[str, torch.Tensor] = {}
    io["x"] = _randn(gen, T, s.H)
    io["kcache"] = torch.full((B, s.nkv, Lcap, s.d), tail_fill, dtype=torch.bfloat16)
    io["vcache"] = torch.full((B, s.nkv, Lcap, s.d), tail_fill, dtype=torch.bfloat16)
    cu = [0]
    pos: List[int] = []
    sid: List[int] = []
    for b, n in enumerate(seq_tokens):
        cu.append(cu[-1] + int(n))
        pos.extend(range(int(n)))
        sid.extend([b] * int(n))
    io["cu_seqlens"] = torch.tensor(cu, dtype=torch.int32)
    io["pos"] = torch.tensor(pos, dtype=torch.int32)
    io["seq_id"] = torch.tensor(sid, dtype=torch.int32)
    io["seq_lens"] = torch.tensor([int(n) for n in seq_tokens], dtype=torch.int32)
    return io


def draw_ctx_lens(wl: Workload, gen: torch.Generator) -> List[int]:
    if wl.ctx_range is not None:
        lo, hi = wl.ctx_range
        return [int(v) for v in torch.randint(lo, hi + 1, (wl.B,), generator=gen)]
    return [wl.ctx] * wl.B


def build(wl: Workload, seed: Optional[int] = None, tail_fill: float = 0.0,
          ctx_lens: Optional[Sequence[int]] = None):
    """Return (weights, io, ctx_lens) for a named workload, all CPU tensors."""
    gen = torch.Generator().manual_seed(wl.seed if seed is None else seed)
    if wl.mode == "decode":
        lens = list(ctx_lens) if ctx_lens is not None else draw_ctx_lens(wl, gen)
        weights = make_weights(wl.shape, gen)
        io = make_decode_io(wl.shape, lens, gen, tail_fill=tail_fill)
    else:
        lens = [wl.seq_tokens] * wl.B
        weights = make_weights(wl.shape, gen)
        io = make_prefill_io(wl.shape, lens, gen, tail_fill=tail_fill)
    return weights, io, lens


def micro_batches(wl: Workload) -> List[range]:
    """Sequences [i*B/n, (i+1)*B/n) in index order, no length sorting."""
    per = wl.B // wl.n_micro
    return [range(i * per, (i + 1) * per) for i in range(wl.n_micro)]


def scaled(wl: Workload, **kw) -> Workload:
    """A smaller/larger variant of a named workload (tests use it for quick cases)."""
    return replace(wl, **kw)


def randn_bf16(gen: torch.Generator, *shape, std: float = 1.0, mean: float = 0.0) -> torch.Tensor:
    """A seeded N(mean, std) tensor rounded once to bf16 (for per-kernel test inputs)."""
    return _randn(gen, *shape, std=std, mean=mean)
