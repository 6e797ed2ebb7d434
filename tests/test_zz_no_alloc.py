"""The entry point that allocates nothing (ts_attention_decode_static: split-KV partials in the library's own
device array) against the entry point it is a variant of (ts_attention_decode with a caller workspace): two calls
in a row, the second with a smaller input, both bit-identical to the workspace form and within the stated
tolerance of the oracle."""
import math

import numpy as np
import pytest
import torch

import workloads as WL
from oracle import decoder_layer as O
from parity import assert_close, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2604_10180_amd import binding
    return binding


def _case(B, seed, lens, nq, nkv, d, poison):
    gen = torch.Generator().manual_seed(seed)
    Bs, Lcap = len(lens), max(lens)
    q = WL.randn_bf16(gen, Bs, nq, d)
    kc = torch.full((Bs, nkv, Lcap, d), float("nan"), dtype=torch.bfloat16)
    vc = torch.full((Bs, nkv, Lcap, d), float("nan"), dtype=torch.bfloat16)
    for b, L in enumerate(lens):
        kc[b, :, :L] = WL.randn_bf16(gen, nkv, L, d)
        vc[b, :, :L] = WL.randn_bf16(gen, nkv, L, d)
    sl = torch.tensor(lens, dtype=torch.int32)
    scale = 1.0 / math.sqrt(d)
    qd, kd, vd, sd = q.to(DEV), kc.to(DEV), vc.to(DEV), sl.to(DEV)
    need = B.ts_attention_decode_workspace_bytes(Bs, nq, nkv, d, Lcap)
    assert 0 < need <= B.ts_attention_decode_static_limit()
    ws = torch.full((need,), poison, dtype=torch.uint8, device=DEV)
    want = torch.zeros(Bs, nq, d, dtype=torch.bfloat16, device=DEV)
    B.ts_attention_decode(qd, kd, vd, sd, want, Bs, nq, nkv, d, Lcap, scale, ws)
    got = torch.zeros(Bs, nq, d, dtype=torch.bfloat16, device=DEV)
    B.ts_attention_decode_static(qd, kd, vd, sd, got, Bs, nq, nkv, d, Lcap, scale)
    torch.cuda.synchronize()
    assert torch.equal(got, want), "static-scratch form differs from the workspace form"
    ref = O.attention_decode(WL.as_f64(q), WL.as_f32(torch.nan_to_num(kc)), WL.as_f32(torch.nan_to_num(vc)), np.array(lens), scale)
    assert_close(to_np(got), ref, f"ts_attention_decode_static seed {seed}")


def test_static_scratch_decode_attention_two_calls_second_smaller(B):
    # five, three, two and one chunks per sequence, then a smaller call whose partials land on top of the first's
    _case(B, 31, [9000, 4097, 2300, 100, 1, 6500], nq=16, nkv=2, d=128, poison=0xFF)
    _case(B, 32, [4500, 70, 2200], nq=8, nkv=2, d=64, poison=0x7F)
    # rejected before anything is enqueued when the partials do not fit the built-in array
    with pytest.raises(B.TesseraError) as e:
        B.ts_attention_decode_static(16, 16, 16, 16, 16, 64, 128, 8, 128, 1 << 20, 0.1, stream=0)
    assert e.value.code == B.TS_ERR_WORKSPACE
