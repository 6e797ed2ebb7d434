"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and
rejects bad arguments before touching the GPU.  No compute calls."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    so = os.path.join(ROOT, "paper_2604_10180_amd", "libtessera.so")
    if not os.path.exists(so):
        import __graft_entry__
        __graft_entry__.build()
    from paper_2604_10180_amd import binding
    return binding


def test_header_symbols_all_exported(B):
    hdr = open(os.path.join(ROOT, "include", "tessera.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ts_[a-z0-9_]+)\s*\(", hdr))
    assert declared, "no declarations found"
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name), f"{name} not exported"


def test_version_and_strerror(B):
    assert "gfx950" in B.ts_version()
    assert B.ts_strerror(0) == "ok" and "workspace" in B.ts_strerror(B.TS_ERR_WORKSPACE)


def test_argument_errors_without_gpu(B):
    with pytest.raises(B.TesseraError) as e:
        B.ts_rmsnorm(None, None, None, 4, 256, 1e-5, stream=0)
    assert e.value.code == B.TS_ERR_INVALID_ARG and "null" in e.value.detail
    with pytest.raises(B.TesseraError) as e:
        B.ts_rmsnorm(16, 16, 16, 4, 250, 1e-5, stream=0)
    assert e.value.code == B.TS_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(B.TesseraError) as e:
        B.ts_rmsnorm(8, 16, 16, 4, 256, 1e-5, stream=0)          # misaligned
    assert e.value.code == B.TS_ERR_INVALID_ARG
    with pytest.raises(B.TesseraError) as e:
        B.ts_gemm_bf16(16, 16, None, 16, 4, 64, 100, stream=0)   # K % 8 != 0
    assert e.value.code == B.TS_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(B.TesseraError) as e:
        B.ts_attention_decode(16, 16, 16, 16, 16, 2, 6, 4, 128, 64, 0.1, stream=0)   # nq % nkv
    assert e.value.code == B.TS_ERR_INVALID_ARG
    with pytest.raises(B.TesseraError) as e:
        B.ts_attention_decode(16, 16, 16, 16, 16, 2, 8, 2, 96, 64, 0.1, stream=0)    # head dim
    assert e.value.code == B.TS_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(B.TesseraError) as e:
        B.ts_moe_route(16, 4, 8, 9, 16, 16, 16, 16, 16, stream=0)                      # k > E
    assert e.value.code == B.TS_ERR_INVALID_ARG
    with pytest.raises(B.TesseraError) as e:
        B.ts_pipeline_set_link_slowdown(None, 2)                                        # no pipeline
    assert e.value.code == B.TS_ERR_INVALID_ARG
    # T == 0 is a no-op that never reaches the GPU
    B.ts_rmsnorm(None, None, None, 0, 256, 1e-5, stream=0)
    B.ts_swiglu(None, None, 0, 64, stream=0)


def test_workspace_errors_and_sizes(B):
    # split-K projection shapes need scratch; large-row shapes do not
    assert B.ts_gemm_workspace_bytes(64, 4096, 4096) > 0
    assert B.ts_gemm_workspace_bytes(8192, 4096, 4096) == 0
    with pytest.raises(B.TesseraError) as e:
        B.ts_gemm_bf16(16, 16, None, 16, 64, 4096, 4096, ws=None, stream=0)
    assert e.value.code == B.TS_ERR_WORKSPACE
    assert B.ts_attention_decode_workspace_bytes(64, 32, 8, 128, 2049) >= 64 * 32 * 130 * 4
    with pytest.raises(B.TesseraError) as e:
        B.ts_attention_decode(16, 16, 16, 16, 16, 2, 8, 2, 128, 64, 0.1, ws=None, stream=0)
    assert e.value.code == B.TS_ERR_WORKSPACE


def test_layer_planning_host_only(B):
    from workloads import CONFIGS
    for name, wl in CONFIGS.items():
        desc = B.make_desc(wl.shape, Lcap=4096, mode=wl.mode)
        T = 8 if wl.mode == "decode" else 64
        total = B.ts_layer_workspace_bytes(desc, T, 8)
        assert total > 0
        nb = B.TS_NB_MOE if wl.shape.E else B.TS_NB_DENSE
        spans = []
        for i in range(nb):
            off, nbytes = B.ts_layer_boundary(desc, T, 8, i)
            assert nbytes > 0
            if off is not None:
                assert off % 256 == 0 and off + nbytes <= total
                spans.append((off, off + nbytes))
            else:
                assert i == nb - 1
        spans.sort()
        assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:])), "boundary buffers overlap"
        offs = B.ts_pipeline_boundary_layout(desc, T, 8, ~0)
        assert len(offs) == nb + 1 and offs == sorted(offs)
        assert B.ts_pipeline_slot_stride(desc, T, 8, ~0) >= offs[-1]
        sel = B.ts_pipeline_boundary_layout(desc, T, 8, 0b1001)
        assert len(sel) == 3 and sel[1] == T * wl.shape.H * 2
    bad = B.make_desc(CONFIGS["tiny"].shape, Lcap=16, mode="decode")
    bad.d = 96
    assert B.ts_layer_workspace_bytes(bad, 4, 4) == 0
    with pytest.raises(B.TesseraError):
        B.ts_layer_boundary(bad, 4, 4, 0)


def test_pipeline_workspace_slot_is_the_largest_plan_not_the_plan_of_the_largest_micro_batch(B):
    """The layer's workspace size is not monotone in the row count (split-K and split-KV plans change form), and
    every micro-batch lays its slot out with its own plan: the slot must hold the largest of them.  All of it is
    checked before the first HIP call, so it runs on a host without a GPU (the fake pointers are never used)."""
    from workloads import CONFIGS
    for name in ("8b_decode", "70b_pipeline"):
        s = CONFIGS[name].shape
        desc = B.make_desc(s, Lcap=4096, mode="decode")
        sizes = {T: B.ts_layer_workspace_bytes(desc, T, T) for T in range(1, 130)}
        inversions = [T for T in range(1, 129) if sizes[T] > sizes[T + 1]]
        for T in range(1, 129):
            slot = B.ts_pipeline_workspace_slot_bytes(desc, [T + 1, T], [T + 1, T])
            assert slot % 256 == 0 and slot >= sizes[T] and slot >= sizes[T + 1]
            assert slot == max((sizes[T] + 255) // 256 * 256, (sizes[T + 1] + 255) // 256 * 256)
        if not inversions:
            continue
        T = inversions[0]           # plan(T) > plan(T + 1)
        pipe = B.ts_pipeline_create(desc, 2)
        try:
            fake = 4096
            wts = B.LayerWeights(*([fake] * 8), 0)
            mbs = [B.LayerIO(fake, fake, fake, fake, fake, None, fake, fake, t, t, 0) for t in (T + 1, T)]

            class Buf:   # stands in for a device buffer of a given size at a fake address
                def __init__(self, n):
                    self.n = n
                def data_ptr(self):
                    return fake
                def numel(self):
                    return self.n
                def element_size(self):
                    return 1
            too_small = 2 * ((sizes[T + 1] + 255) // 256 * 256)      # two slots sized for the larger micro-batch only
            assert too_small < 2 * B.ts_pipeline_workspace_slot_bytes(desc, [T + 1, T], [T + 1, T])
            with pytest.raises(B.TesseraError) as e:
                B.ts_pipeline_step(pipe, wts, mbs, [0, 0], 0, 0, None, None, Buf(too_small))
            assert e.value.code == B.TS_ERR_WORKSPACE
        finally:
            B.ts_pipeline_destroy(pipe)
    assert inversions or name != "70b_pipeline"
    assert B.ts_pipeline_workspace_slot_bytes(desc, [], []) == 0
