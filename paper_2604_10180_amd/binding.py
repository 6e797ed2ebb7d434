"""ctypes binding of libtessera.so: same names as the C ABI, torch tensors in, status checked.

PyTorch is used for device memory and streams only.  Pointers are taken with
`data_ptr()`; no tensor is copied, converted or computed on here.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtessera.so")

TS_OK, TS_ERR_INVALID_ARG, TS_ERR_UNSUPPORTED_SHAPE, TS_ERR_WORKSPACE, TS_ERR_HIP = 0, -1, -2, -3, -4
TS_MODE_DECODE, TS_MODE_PREFILL = 0, 1
(TS_B_H1, TS_B_QKV, TS_B_ATTN, TS_B_X2, TS_B_H2, TS_B_GATE_UP, TS_B_ACT) = range(7)
TS_B_OUT_DENSE, TS_NB_DENSE = 7, 8
TS_B_Y_MOE, TS_B_OUT_MOE, TS_NB_MOE = 7, 8, 9

EXPORTS = [
    "ts_strerror", "ts_last_error", "ts_version", "ts_profile_begin", "ts_profile_end", "ts_rmsnorm", "ts_gemm_workspace_bytes", "ts_gemm_bf16",
    "ts_gemm_bf16_f32out", "ts_rope", "ts_rope_table", "ts_attention_decode_workspace_bytes",
    "ts_attention_decode", "ts_attention_decode_static", "ts_attention_decode_static_limit", "ts_attention_prefill", "ts_swiglu", "ts_moe_route", "ts_moe_gemm", "ts_moe_combine",
    "ts_layer_workspace_bytes", "ts_layer_boundary", "ts_layer_moe_buffers", "ts_layer_node_accesses", "ts_layer_forward",
    "ts_pipeline_create", "ts_pipeline_destroy", "ts_pipeline_boundary_layout", "ts_pipeline_slot_stride",
    "ts_pipeline_workspace_slot_bytes",
    "ts_pipeline_step", "ts_pipeline_kv_delta_stride", "ts_pipeline_set_kv_delta", "ts_pipeline_set_link_slowdown", "ts_ddg_build", "ts_layer_ddg", "ts_layer_node_name", "ts_layer_cut_mask", "ts_plan_policy", "ts_plan_policy_bounded", "ts_plan_lower_bound",
    "ts_monitor_create", "ts_monitor_destroy", "ts_monitor_record", "ts_monitor_advance",
]


class TesseraError(RuntimeError):
    def __init__(self, code: int, detail: str):
        super().__init__(f"tessera error {code}: {detail}")
        self.code = code
        self.detail = detail


class LayerDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("H", "nq", "nkv", "d", "F", "E", "k", "Lcap", "mode")] + \
               [("eps", C.c_float), ("rope_base", C.c_float)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("gamma1", "w_qkv", "w_o", "gamma2", "w_router", "w_gate_up", "w_down",
                                          "rope_cos_sin")] + [("rope_table_len", C.c_int32)]


class LayerIO(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("x", "out", "pos", "seq_id", "seq_lens", "cu_seqlens", "kcache", "vcache")] + \
               [("T", C.c_int32), ("B", C.c_int32), ("max_seqlen", C.c_int32)]


class LayerAccess(C.Structure):
    _fields_ = [("buffer", C.c_int32), ("kind", C.c_int32), ("offset", C.c_uint64), ("extent", C.c_uint64),
                ("bytes", C.c_uint64), ("iter_advance", C.c_int64)]


TS_BUF_WORKSPACE, TS_BUF_X, TS_BUF_OUT, TS_BUF_KCACHE, TS_BUF_VCACHE = range(5)
TS_ACC_READ, TS_ACC_WRITE, TS_ACC_PRIVATE = range(3)


class Access(C.Structure):
    _fields_ = [("addr", C.c_uint64), ("extent", C.c_uint64), ("bytes", C.c_uint64), ("iter_advance", C.c_int64)]


class KernelIO(C.Structure):
    _fields_ = [("reads", C.POINTER(Access)), ("writes", C.POINTER(Access)), ("n_reads", C.c_int32),
                ("n_writes", C.c_int32)]


class DdgEdge(C.Structure):
    _fields_ = [("src", C.c_int32), ("dst", C.c_int32), ("bytes", C.c_uint64), ("cross_iteration", C.c_int32),
                ("reserved", C.c_int32)]


class PlanProblem(C.Structure):
    _fields_ = [("n_kernels", C.c_int32), ("n_gpus", C.c_int32), ("n_edges", C.c_int32), ("reserved", C.c_int32),
                ("t", C.POINTER(C.c_double)), ("edges", C.POINTER(DdgEdge)), ("bw", C.POINTER(C.c_double)),
                ("lat", C.POINTER(C.c_double))]


TS_PLAN_THROUGHPUT, TS_PLAN_LATENCY = 0, 1
TS_PIPE_COPY_SIDE_STREAM, TS_PIPE_COPY_SERIALISED, TS_PIPE_COPY_COALESCED, TS_PIPE_COPY_COALESCED_HALVES = 0, 1, 2, 3


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_10180_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    for n in ("ts_strerror", "ts_last_error", "ts_version"):
        getattr(lib, n).restype = C.c_char_p
    for n in ("ts_gemm_workspace_bytes", "ts_attention_decode_workspace_bytes", "ts_layer_workspace_bytes",
              "ts_pipeline_slot_stride", "ts_pipeline_kv_delta_stride", "ts_pipeline_workspace_slot_bytes",
              "ts_attention_decode_static_limit"):
        getattr(lib, n).restype = C.c_size_t
    lib.ts_pipeline_destroy.restype = None
    lib.ts_layer_node_name.restype = C.c_char_p
    lib.ts_monitor_destroy.restype = None
    return lib


lib = _load()

_i, _f, _p, _z, _u64 = C.c_int, C.c_float, C.c_void_p, C.c_size_t, C.c_uint64
lib.ts_strerror.argtypes = [_i]
lib.ts_profile_begin.argtypes = [C.POINTER(_p), C.POINTER(C.c_char_p), _i]
lib.ts_profile_end.argtypes = []
lib.ts_rmsnorm.argtypes = [_p, _p, _p, _i, _i, _f, _p]
lib.ts_gemm_workspace_bytes.argtypes = [_i, _i, _i]
lib.ts_gemm_bf16.argtypes = [_p, _p, _p, _p, _i, _i, _i, _p, _z, _p]
lib.ts_gemm_bf16_f32out.argtypes = [_p, _p, _p, _i, _i, _i, _p, _z, _p]
lib.ts_rope.argtypes = [_p, _p, _p, _i, _i, _p, _p, _p, _i, _p, _p, _i, _i, _i, _i, _i, _f, _p]
lib.ts_rope_table.argtypes = [_p, _i, _i, _f]
lib.ts_attention_decode_workspace_bytes.argtypes = [_i, _i, _i, _i, _i]
lib.ts_attention_decode.argtypes = [_p, _p, _p, _p, _p, _i, _i, _i, _i, _i, _f, _p, _z, _p]
lib.ts_attention_decode_static.argtypes = [_p, _p, _p, _p, _p, _i, _i, _i, _i, _i, _f, _p]
lib.ts_attention_decode_static_limit.argtypes = []
lib.ts_attention_prefill.argtypes = [_p, _p, _p, _i, _i, _p, _p, _i, _i, _i, _i, _i, _i, _f, _i, _p]
lib.ts_swiglu.argtypes = [_p, _p, _i, _i, _p]
lib.ts_moe_route.argtypes = [_p, _i, _i, _i, _p, _p, _p, _p, _p, _p]
lib.ts_moe_gemm.argtypes = [_p, _p, _i, _p, _p, _p, _i, _i, _i, _i, _p]
lib.ts_moe_combine.argtypes = [_p, _p, _p, _p, _p, _p, _i, _i, _i, _p]
lib.ts_layer_workspace_bytes.argtypes = [C.POINTER(LayerDesc), _i, _i]
lib.ts_layer_boundary.argtypes = [C.POINTER(LayerDesc), _i, _i, _i, C.POINTER(_z), C.POINTER(_z)]
lib.ts_layer_moe_buffers.argtypes = [C.POINTER(LayerDesc), _i, _i, C.POINTER(_z)]
lib.ts_layer_node_accesses.argtypes = [C.POINTER(LayerDesc), _i, _i, _i, _i, C.POINTER(LayerAccess), _i, C.POINTER(_i)]
lib.ts_layer_forward.argtypes = [C.POINTER(LayerDesc), C.POINTER(LayerWeights), C.POINTER(LayerIO), _p, _z, _p]
lib.ts_pipeline_create.argtypes = [C.POINTER(LayerDesc), _i, C.POINTER(_p)]
lib.ts_pipeline_destroy.argtypes = [_p]
lib.ts_pipeline_boundary_layout.argtypes = [C.POINTER(LayerDesc), _i, _i, _u64, C.POINTER(_z), C.POINTER(_i)]
lib.ts_pipeline_slot_stride.argtypes = [C.POINTER(LayerDesc), _i, _i, _u64]
lib.ts_pipeline_kv_delta_stride.argtypes = [C.POINTER(LayerDesc), _i]
lib.ts_pipeline_workspace_slot_bytes.argtypes = [C.POINTER(LayerDesc), C.POINTER(C.c_int32), C.POINTER(C.c_int32), _i]
lib.ts_pipeline_set_kv_delta.argtypes = [_p, _p, _p, _p, _z]
lib.ts_pipeline_set_link_slowdown.argtypes = [_p, C.c_int]
lib.ts_pipeline_step.argtypes = [_p, C.POINTER(LayerWeights), C.POINTER(LayerIO), _i, C.POINTER(_p), _p, _u64, _i,
                                 _p, _p, _z, _p, _z]
lib.ts_ddg_build.argtypes = [C.POINTER(KernelIO), _i, C.POINTER(DdgEdge), _i, C.POINTER(_i)]
lib.ts_layer_ddg.argtypes = [C.POINTER(LayerDesc), _i, _i, _i, _i, C.POINTER(DdgEdge), _i, C.POINTER(_i)]
lib.ts_layer_node_name.argtypes = [C.POINTER(LayerDesc), _i]
lib.ts_layer_cut_mask.argtypes = [C.POINTER(LayerDesc), C.POINTER(C.c_int32), C.POINTER(_u64)]
lib.ts_plan_policy.argtypes = [C.POINTER(PlanProblem), _i, C.c_int64, C.POINTER(C.c_int32), C.POINTER(C.c_double),
                               C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(_i)]
lib.ts_plan_policy_bounded.argtypes = [C.POINTER(PlanProblem), _i, C.c_int64, C.c_double, C.POINTER(C.c_int32),
                                       C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double),
                                       C.POINTER(C.c_double), C.POINTER(_i)]
lib.ts_plan_lower_bound.argtypes = [C.POINTER(PlanProblem), _i, C.POINTER(C.c_double)]
lib.ts_monitor_create.argtypes = [C.c_double, C.c_double, _i, C.POINTER(_p)]
lib.ts_monitor_destroy.argtypes = [_p]
lib.ts_monitor_record.argtypes = [_p, C.c_double, C.c_double, C.POINTER(C.c_double), _i, C.c_double]
lib.ts_monitor_advance.argtypes = [_p, C.c_double, C.POINTER(_i), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                   C.POINTER(C.c_double)]


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(s) -> Optional[int]:
    if s is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def _check(rc: int) -> None:
    if rc != TS_OK:
        raise TesseraError(rc, lib.ts_last_error().decode())


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def ts_version() -> str:
    return lib.ts_version().decode()


def ts_strerror(code: int) -> str:
    return lib.ts_strerror(code).decode()


def ts_last_error() -> str:
    return lib.ts_last_error().decode()


def ts_rmsnorm(x, gamma, y, T: int, H: int, eps: float, stream=None) -> None:
    _check(lib.ts_rmsnorm(_ptr(x), _ptr(gamma), _ptr(y), T, H, eps, _stream(stream)))


def ts_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return lib.ts_gemm_workspace_bytes(M, N, K)


def ts_gemm_bf16(A, W, residual, Cout, M: int, N: int, K: int, ws=None, stream=None) -> None:
    _check(lib.ts_gemm_bf16(_ptr(A), _ptr(W), _ptr(residual), _ptr(Cout), M, N, K, _ptr(ws), _nbytes(ws),
                            _stream(stream)))


def ts_gemm_bf16_f32out(A, W, Cout, M: int, N: int, K: int, ws=None, stream=None) -> None:
    _check(lib.ts_gemm_bf16_f32out(_ptr(A), _ptr(W), _ptr(Cout), M, N, K, _ptr(ws), _nbytes(ws), _stream(stream)))


def ts_rope(q, k, v, q_stride: int, kv_stride: int, pos, seq_id, cos_sin, table_len: int, kcache, vcache, T: int,
            nq: int, nkv: int, d: int, Lcap: int, base: float, stream=None) -> None:
    _check(lib.ts_rope(_ptr(q), _ptr(k), _ptr(v), q_stride, kv_stride, _ptr(pos), _ptr(seq_id), _ptr(cos_sin),
                       table_len, _ptr(kcache), _ptr(vcache), T, nq, nkv, d, Lcap, base, _stream(stream)))


def ts_rope_table(table_host: torch.Tensor, table_len: int, d: int, base: float) -> None:
    """table_host: CPU float32 tensor [table_len, d], filled in place."""
    assert not table_host.is_cuda and table_host.dtype == torch.float32 and table_host.numel() >= table_len * d
    _check(lib.ts_rope_table(table_host.data_ptr(), table_len, d, base))


def ts_attention_decode_workspace_bytes(B: int, nq: int, nkv: int, d: int, Lcap: int) -> int:
    return lib.ts_attention_decode_workspace_bytes(B, nq, nkv, d, Lcap)


def ts_attention_decode(q, kcache, vcache, seq_lens, out, B: int, nq: int, nkv: int, d: int, Lcap: int, scale: float,
                        ws=None, stream=None) -> None:
    _check(lib.ts_attention_decode(_ptr(q), _ptr(kcache), _ptr(vcache), _ptr(seq_lens), _ptr(out), B, nq, nkv, d, Lcap,
                                   scale, _ptr(ws), _nbytes(ws), _stream(stream)))


def ts_attention_decode_static_limit() -> int:
    return lib.ts_attention_decode_static_limit()


def ts_attention_decode_static(q, kcache, vcache, seq_lens, out, B: int, nq: int, nkv: int, d: int, Lcap: int,
                               scale: float, stream=None) -> None:
    _check(lib.ts_attention_decode_static(_ptr(q), _ptr(kcache), _ptr(vcache), _ptr(seq_lens), _ptr(out), B, nq, nkv, d,
                                          Lcap, scale, _stream(stream)))


def ts_attention_prefill(q, k, v, q_stride: int, kv_stride: int, cu_seqlens, out, S: int, T: int, max_seqlen: int,
                         nq: int, nkv: int, d: int, scale: float, causal: bool = True, stream=None) -> None:
    _check(lib.ts_attention_prefill(_ptr(q), _ptr(k), _ptr(v), q_stride, kv_stride, _ptr(cu_seqlens), _ptr(out), S, T,
                                    max_seqlen, nq, nkv, d, scale, 1 if causal else 0, _stream(stream)))


def ts_swiglu(gate_up, out, T: int, F: int, stream=None) -> None:
    _check(lib.ts_swiglu(_ptr(gate_up), _ptr(out), T, F, _stream(stream)))


def ts_moe_route(logits, T: int, E: int, k: int, topk_idx, topk_w, counts, offsets, perm, stream=None) -> None:
    _check(lib.ts_moe_route(_ptr(logits), T, E, k, _ptr(topk_idx), _ptr(topk_w), _ptr(counts), _ptr(offsets),
                            _ptr(perm), _stream(stream)))


def ts_moe_gemm(A, row_map, row_div: int, W, offsets, Cout, rows: int, E: int, N: int, K: int, stream=None) -> None:
    _check(lib.ts_moe_gemm(_ptr(A), _ptr(row_map), row_div, _ptr(W), _ptr(offsets), _ptr(Cout), rows, E, N, K,
                           _stream(stream)))


def ts_moe_combine(y, perm, topk_w, residual, out, scratch_inv, T: int, k: int, H: int, stream=None) -> None:
    _check(lib.ts_moe_combine(_ptr(y), _ptr(perm), _ptr(topk_w), _ptr(residual), _ptr(out), _ptr(scratch_inv), T, k, H,
                              _stream(stream)))


# ---------------------------------------------------------------- layer / pipeline marshalling
def make_desc(shape, Lcap: int, mode: str) -> LayerDesc:
    return LayerDesc(H=shape.H, nq=shape.nq, nkv=shape.nkv, d=shape.d, F=shape.F, E=shape.E, k=shape.k, Lcap=Lcap,
                     mode=TS_MODE_DECODE if mode == "decode" else TS_MODE_PREFILL, eps=shape.eps,
                     rope_base=shape.rope_base)


def make_weights(w: dict, rope_table=None) -> LayerWeights:
    return LayerWeights(gamma1=_ptr(w["gamma1"]), w_qkv=_ptr(w["w_qkv"]), w_o=_ptr(w["w_o"]), gamma2=_ptr(w["gamma2"]),
                        w_router=_ptr(w.get("w_router")), w_gate_up=_ptr(w["w_gate_up"]), w_down=_ptr(w["w_down"]),
                        rope_cos_sin=_ptr(rope_table), rope_table_len=0 if rope_table is None else rope_table.shape[0])


def make_io(io: dict, out, T: int, B: int, max_seqlen: int = 0) -> LayerIO:
    return LayerIO(x=_ptr(io["x"]), out=_ptr(out), pos=_ptr(io["pos"]), seq_id=_ptr(io["seq_id"]),
                   seq_lens=_ptr(io.get("seq_lens")), cu_seqlens=_ptr(io.get("cu_seqlens")), kcache=_ptr(io["kcache"]),
                   vcache=_ptr(io["vcache"]), T=T, B=B, max_seqlen=max_seqlen)


def ts_layer_workspace_bytes(desc: LayerDesc, T: int, B: int) -> int:
    return lib.ts_layer_workspace_bytes(C.byref(desc), T, B)


def ts_layer_boundary(desc: LayerDesc, T: int, B: int, index: int):
    off, nb = _z(), _z()
    _check(lib.ts_layer_boundary(C.byref(desc), T, B, index, C.byref(off), C.byref(nb)))
    o = off.value
    return (None if o == C.c_size_t(-1).value else o), nb.value


def ts_layer_moe_buffers(desc: LayerDesc, T: int, B: int):
    arr = (_z * 6)()
    _check(lib.ts_layer_moe_buffers(C.byref(desc), T, B, arr))
    return list(arr)


def ts_layer_node_accesses(desc: LayerDesc, T: int, B: int, kv_len: int, node: int):
    """[(buffer, kind, offset, extent, bytes, iter_advance)] declared for one node of the layer."""
    n = _i()
    rc = lib.ts_layer_node_accesses(C.byref(desc), T, B, kv_len, node, None, 0, C.byref(n))
    if rc not in (TS_OK, TS_ERR_WORKSPACE):
        _check(rc)
    arr = (LayerAccess * max(1, n.value))()
    _check(lib.ts_layer_node_accesses(C.byref(desc), T, B, kv_len, node, arr, n.value, C.byref(n)))
    return [(a.buffer, a.kind, a.offset, a.extent, a.bytes, a.iter_advance) for a in arr[: n.value]]


def ts_layer_forward(desc: LayerDesc, weights: LayerWeights, io: LayerIO, ws, stream=None) -> None:
    _check(lib.ts_layer_forward(C.byref(desc), C.byref(weights), C.byref(io), _ptr(ws), _nbytes(ws), _stream(stream)))


def ts_pipeline_create(desc: LayerDesc, max_micro_batches: int) -> int:
    h = _p()
    _check(lib.ts_pipeline_create(C.byref(desc), max_micro_batches, C.byref(h)))
    return h.value


def ts_pipeline_destroy(handle: int) -> None:
    lib.ts_pipeline_destroy(handle)


def ts_pipeline_boundary_layout(desc: LayerDesc, T: int, B: int, mask: int):
    offs = (_z * (TS_NB_MOE + 1))()
    n = _i()
    _check(lib.ts_pipeline_boundary_layout(C.byref(desc), T, B, mask & (2 ** 64 - 1), offs, C.byref(n)))
    return list(offs[: n.value + 1])


def ts_pipeline_slot_stride(desc: LayerDesc, T: int, B: int, mask: int) -> int:
    return lib.ts_pipeline_slot_stride(C.byref(desc), T, B, mask & (2 ** 64 - 1))


def ts_pipeline_workspace_slot_bytes(desc: LayerDesc, Ts: Sequence[int], Bs: Sequence[int]) -> int:
    n = len(Ts)
    return lib.ts_pipeline_workspace_slot_bytes(C.byref(desc), (C.c_int32 * n)(*Ts), (C.c_int32 * n)(*Bs), n)


def ts_pipeline_kv_delta_stride(desc: LayerDesc, T: int) -> int:
    return lib.ts_pipeline_kv_delta_stride(C.byref(desc), T)


def ts_pipeline_set_kv_delta(handle: int, delta_stream, dev_slots, host_slots) -> None:
    """dev_slots / host_slots: uint8 tensors of equal size (None, None switches the replication off)."""
    if dev_slots is None and host_slots is None:
        _check(lib.ts_pipeline_set_kv_delta(handle, None, None, None, 0))
        return
    _check(lib.ts_pipeline_set_kv_delta(handle, _stream(delta_stream), _ptr(dev_slots), _ptr(host_slots),
                                        min(_nbytes(dev_slots), _nbytes(host_slots))))


def ts_pipeline_set_link_slowdown(handle: int, factor: int) -> None:
    _check(lib.ts_pipeline_set_link_slowdown(handle, factor))


def ts_pipeline_step(handle: int, weights: LayerWeights, mbs: Sequence[LayerIO], compute_streams, copy_stream,
                     mask: int, dev_staging, pinned_host, ws, copy_on_compute_stream: bool = False,
                     copy_mode: Optional[int] = None) -> None:
    arr = (LayerIO * len(mbs))(*mbs)
    cs = (_p * 2)(_stream(compute_streams[0]), _stream(compute_streams[1]))
    _check(lib.ts_pipeline_step(handle, C.byref(weights), arr, len(mbs), cs, _stream(copy_stream),
                                mask & (2 ** 64 - 1),
                                (1 if copy_on_compute_stream else 0) if copy_mode is None else copy_mode, _ptr(dev_staging),
                                _ptr(pinned_host), _nbytes(dev_staging), _ptr(ws), _nbytes(ws)))


def _edges_out(call):
    """Run an edge-producing call, growing the edge array until it fits.  Returns [(src, dst, bytes, cross)]."""
    cap = 256
    while True:
        arr, n = (DdgEdge * cap)(), _i()
        rc = call(arr, cap, C.byref(n))
        if rc == TS_ERR_WORKSPACE and n.value > cap:
            cap = n.value
            continue
        _check(rc)
        return [(arr[i].src, arr[i].dst, arr[i].bytes, arr[i].cross_iteration) for i in range(n.value)]


def _access_array(accesses):
    arr = (Access * max(1, len(accesses)))()
    for i, a in enumerate(accesses):
        arr[i] = Access(a[0], a[1], a[2], a[3] if len(a) > 3 else 0)
    return arr


def ts_ddg_build(kernels):
    """kernels[k] = {"reads": [(addr, extent, bytes[, iter_advance])...], "writes": [...]} in execution order."""
    keep = []
    ks = (KernelIO * max(1, len(kernels)))()
    for i, k in enumerate(kernels):
        r, w = _access_array(k["reads"]), _access_array(k["writes"])
        keep += [r, w]
        ks[i] = KernelIO(r, w, len(k["reads"]), len(k["writes"]))
    return _edges_out(lambda arr, cap, n: lib.ts_ddg_build(ks, len(kernels), arr, cap, n))


def ts_layer_ddg(desc: LayerDesc, T: int, B: int, kv_len: int, n_layers: int = 1):
    return _edges_out(lambda arr, cap, n: lib.ts_layer_ddg(C.byref(desc), T, B, kv_len, n_layers, arr, cap, n))


def ts_layer_node_name(desc: LayerDesc, node: int) -> Optional[str]:
    r = lib.ts_layer_node_name(C.byref(desc), node)
    return None if r is None else r.decode()


def ts_layer_cut_mask(desc: LayerDesc, placement: Sequence[int]) -> int:
    nb = TS_NB_MOE if desc.E > 0 else TS_NB_DENSE
    if len(placement) != nb + 1:
        raise ValueError(f"placement needs {nb + 1} entries (the layer's nodes, then the consumer of its output)")
    arr, mask = (C.c_int32 * (nb + 1))(*placement), _u64()
    _check(lib.ts_layer_cut_mask(C.byref(desc), arr, C.byref(mask)))
    return mask.value


def _plan_problem(t, edges, bw, lat):
    K, G = len(t), len(t[0])
    flat = lambda m: (C.c_double * (len(m) * len(m[0])))(*[float(v) for row in m for v in row])
    ta = flat(t)
    ea = (DdgEdge * max(1, len(edges)))()
    for i, e in enumerate(edges):
        ea[i] = DdgEdge(e[0], e[1], int(e[2]), e[3] if len(e) > 3 else 0, 0)
    ba, la = (flat(bw) if bw is not None else None), (flat(lat) if lat is not None else None)
    return PlanProblem(K, G, len(edges), 0, ta, ea, ba, la), (ta, ea, ba, la)


def ts_plan_lower_bound(t, edges, bw, lat, objective: int) -> float:
    prob, _keep = _plan_problem(t, edges, bw, lat)
    out = C.c_double()
    _check(lib.ts_plan_lower_bound(C.byref(prob), objective, C.byref(out)))
    return out.value


def ts_plan_policy(t, edges, bw, lat, objective: int, node_limit: int = 0):
    """t: [K][G] seconds; edges: [(src, dst, bytes[, cross])]; bw, lat: [G][G].
    Returns (placement, value, T_g, M_g, proved_optimal)."""
    K, G = len(t), len(t[0])
    prob, _keep = _plan_problem(t, edges, bw, lat)
    place, val, opt = (C.c_int32 * K)(), C.c_double(), _i()
    Tg, Mg = (C.c_double * G)(), (C.c_double * G)()
    _check(lib.ts_plan_policy(C.byref(prob), objective, node_limit, place, C.byref(val), Tg, Mg, C.byref(opt)))
    return list(place), val.value, list(Tg), list(Mg), bool(opt.value)


def ts_plan_policy_bounded(t, edges, bw, lat, objective: int, rel_gap: float, node_limit: int = 0):
    """Returns (placement, value, T_g, M_g, lower_bound, status); status 2 = optimal, 1 = within rel_gap of the
    lower bound, 0 = stopped by the node limit."""
    K, G = len(t), len(t[0])
    prob, _keep = _plan_problem(t, edges, bw, lat)
    place, val, lb, st = (C.c_int32 * K)(), C.c_double(), C.c_double(), _i()
    Tg, Mg = (C.c_double * G)(), (C.c_double * G)()
    _check(lib.ts_plan_policy_bounded(C.byref(prob), objective, node_limit, rel_gap, place, C.byref(val), Tg, Mg,
                                      C.byref(lb), C.byref(st)))
    return list(place), val.value, list(Tg), list(Mg), lb.value, st.value


def ts_monitor_create(window_s: float = 0.3, beta: float = 1.5, initial_policy: int = TS_PLAN_LATENCY) -> int:
    h = _p()
    _check(lib.ts_monitor_create(window_s, beta, initial_policy, C.byref(h)))
    return h.value


def ts_monitor_destroy(handle: int) -> None:
    lib.ts_monitor_destroy(handle)


def ts_monitor_record(handle: int, t_complete: float, request_latency: float, group_latencies: Sequence[float],
                      comm: float) -> None:
    arr = (C.c_double * max(1, len(group_latencies)))(*group_latencies)
    _check(lib.ts_monitor_record(handle, t_complete, request_latency, arr, len(group_latencies), comm))


def ts_monitor_advance(handle: int, now: float):
    """Returns (policy, windows closed, switches, ratio of the last non-empty window)."""
    pol, nwin, nsw, ratio = _i(), C.c_int64(), C.c_int64(), C.c_double()
    _check(lib.ts_monitor_advance(handle, now, C.byref(pol), C.byref(nwin), C.byref(nsw), C.byref(ratio)))
    return pol.value, nwin.value, nsw.value, ratio.value


class KernelProfile:
    """Brackets every library launch on this thread with a pair of timing events.

    with KernelProfile(max_launches) as prof: ...calls...; then prof.durations_ms() after a sync
    returns [(kernel_family_name, milliseconds), ...] in launch order.
    """

    def __init__(self, max_launches: int):
        self.cap = max_launches
        self.events = [torch.cuda.Event(enable_timing=True) for _ in range(2 * max_launches)]
        for e in self.events:          # torch creates the HIP event lazily, on the first record
            e.record()
        torch.cuda.synchronize()
        self._ev = (_p * (2 * max_launches))(*[e.cuda_event for e in self.events])
        self._names = (C.c_char_p * max_launches)()
        self.n = 0

    def __enter__(self):
        _check(lib.ts_profile_begin(self._ev, self._names, self.cap))
        return self

    def __exit__(self, *exc):
        self.n = lib.ts_profile_end()
        return False

    def durations_ms(self):
        torch.cuda.synchronize()
        return [(self._names[i].decode(), self.events[2 * i].elapsed_time(self.events[2 * i + 1]))
                for i in range(self.n)]
