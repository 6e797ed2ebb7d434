"""The kernels against the byte ranges declared for them (ts_layer_node_accesses), the one-GPU counterpart of the
paper's memory access analysis (Sec. 3.1: the analyzer derives the [min, max] range each kernel touches; here the
ranges are declared by hand and the dependency graph is built from them, so the kernels are held to them):

  * writes: the workspace, the residual input, the output and both caches sit between guard bands, and everything
    that no node declares as written (or as its private scratch) is filled with a pattern: after ts_layer_forward
    the guard bands, the pattern, the input and every cache row outside the declared append are untouched;
  * reads: the same call is run with the whole workspace and the unused cache tails filled with NaN patterns and
    with another filler: every declared output is bit-identical, so no kernel reads a byte of the workspace that
    this call has not written first, nor a cache position beyond the declared lengths.
"""
import numpy as np
import pytest
import torch

import workloads as WL

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GUARD = 4096


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2604_10180_amd import binding
    return binding


def guarded(t: torch.Tensor, fill: int):
    """A device copy of `t` with GUARD bytes of `fill` on either side; returns (whole uint8 buffer, view like t)."""
    raw = t.contiguous().view(torch.uint8).reshape(-1)
    big = torch.full((raw.numel() + 2 * GUARD,), fill, dtype=torch.uint8, device=DEV)
    big[GUARD:GUARD + raw.numel()] = raw.to(DEV)
    return big, big[GUARD:GUARD + raw.numel()].view(t.dtype).reshape(t.shape)


def guards_intact(big: torch.Tensor, fill: int) -> bool:
    return bool((big[:GUARD] == fill).all()) and bool((big[-GUARD:] == fill).all())


def run_declared(B, wl, weights, io, ws_fill, tail_fill, use_table=True):
    s = wl.shape
    Lcap = io["kcache"].shape[2]
    T, Bs = io["x"].shape[0], io["kcache"].shape[0]
    desc = B.make_desc(s, Lcap, wl.mode)
    nb = B.TS_NB_MOE if s.E else B.TS_NB_DENSE
    wd = {k: v.to(DEV) for k, v in weights.items()}
    table = None
    if use_table:
        th = torch.empty(Lcap, s.d, dtype=torch.float32)
        B.ts_rope_table(th, Lcap, s.d, s.rope_base)
        table = th.to(DEV)
    kv_len = int(io["seq_lens"][0]) if wl.mode == "decode" else 1
    kc, vc = io["kcache"].clone(), io["vcache"].clone()
    if wl.mode == "decode":          # positions from the appended one on are not part of the input
        kc[:, :, kv_len - 1:] = tail_fill
        vc[:, :, kv_len - 1:] = tail_fill
    else:
        kc[:], vc[:] = tail_fill, tail_fill
    G = 0x3C
    x_big, x = guarded(io["x"], G)
    kc_big, kcd = guarded(kc, G)
    vc_big, vcd = guarded(vc, G)
    out_big, out = guarded(torch.zeros(T, s.H, dtype=torch.bfloat16), G)
    out_big[GUARD:-GUARD] = ws_fill
    ws_bytes = B.ts_layer_workspace_bytes(desc, T, Bs)
    ws_big = torch.full((ws_bytes + 2 * GUARD,), ws_fill, dtype=torch.uint8, device=DEV)
    ws_big[:GUARD], ws_big[-GUARD:] = G, G
    ws = ws_big[GUARD:GUARD + ws_bytes]
    iod = {"x": x, "pos": io["pos"].to(DEV), "seq_id": io["seq_id"].to(DEV), "kcache": kcd, "vcache": vcd}
    for k in ("seq_lens", "cu_seqlens"):
        if k in io:
            iod[k] = io[k].to(DEV)
    max_seqlen = int(io["seq_lens"].max()) if wl.mode == "prefill" else 0
    x_before, kc_before, vc_before = x.clone(), kcd.clone(), vcd.clone()
    B.ts_layer_forward(desc, B.make_weights(wd, table), B.make_io(iod, out, T, Bs, max_seqlen), ws)
    torch.cuda.synchronize()

    # ---- what the nodes declare
    written = {b: None for b in range(5)}
    sizes = {B.TS_BUF_WORKSPACE: ws_bytes, B.TS_BUF_X: x.numel() * 2, B.TS_BUF_OUT: out.numel() * 2,
             B.TS_BUF_KCACHE: kcd.numel() * 2, B.TS_BUF_VCACHE: vcd.numel() * 2}
    for b in sizes:
        written[b] = torch.zeros(sizes[b], dtype=torch.bool, device=DEV)
    outputs = []          # (buffer, offset, extent) of declared writes that carry data (not private scratch)
    for node in range(nb):
        for buf, kind, off, ext, nbytes, adv in B.ts_layer_node_accesses(desc, T, Bs, kv_len, node):
            assert off + ext <= sizes[buf], (node, buf, off, ext, sizes[buf])
            assert nbytes <= ext
            if kind in (B.TS_ACC_WRITE, B.TS_ACC_PRIVATE):
                written[buf][off:off + ext] = True
                if kind == B.TS_ACC_WRITE:
                    outputs.append((buf, off, ext))
    # ---- writes stay inside the declarations
    for big in (x_big, kc_big, vc_big, out_big, ws_big):
        assert guards_intact(big, G), "a guard band was written"
    assert not bool(written[B.TS_BUF_X].any()) and torch.equal(x, x_before), "the residual input was written"
    assert bool((ws[~written[B.TS_BUF_WORKSPACE]] == ws_fill).all()), "workspace bytes outside every declared write changed"
    for cache, before, buf in ((kcd, kc_before, B.TS_BUF_KCACHE), (vcd, vc_before, B.TS_BUF_VCACHE)):
        same = cache.view(torch.uint8).reshape(-1) == before.view(torch.uint8).reshape(-1)
        assert bool(same[~written[buf]].all()), "cache bytes outside the declared append changed"
    assert bool(written[B.TS_BUF_OUT].all())
    bufs = {B.TS_BUF_WORKSPACE: ws, B.TS_BUF_OUT: out.view(torch.uint8).reshape(-1),
            B.TS_BUF_KCACHE: kcd.view(torch.uint8).reshape(-1), B.TS_BUF_VCACHE: vcd.view(torch.uint8).reshape(-1)}
    # prefill declares the hull of the fresh cache rows (whole cache); compare only what it really wrote there
    result = []
    for buf, off, ext in sorted(set(outputs)):
        if wl.mode == "prefill" and buf in (B.TS_BUF_KCACHE, B.TS_BUF_VCACHE):
            cache = kcd if buf == B.TS_BUF_KCACHE else vcd
            n = int(io["seq_lens"].max())
            result.append(((buf, off, ext), cache[:, :, :n].clone()))
        else:
            result.append(((buf, off, ext), bufs[buf][off:off + ext].clone()))
    assert bool(torch.isfinite(out.float()).all()), "non-finite layer output"
    return result


CASES = {
    "tiny": lambda: (WL.CONFIGS["tiny"], {}),
    "small_moe": lambda: (WL.Workload("moe", WL.LayerShape(H=512, nq=8, nkv=2, d=64, F=688, E=8, k=2), "decode", B=48, ctx=300), {}),
    "long_context_merge_in_launch": lambda: (WL.Workload("long", WL.LayerShape(H=256, nq=8, nkv=1, d=128, F=688), "decode", B=3, ctx=9000), {}),
    "8b_decode": lambda: (WL.CONFIGS["8b_decode"], {}),
    "moe_decode": lambda: (WL.CONFIGS["moe_decode"], {}),
    "70b_micro_batch": lambda: (WL.Workload("70b_mb", WL.CONFIGS["70b_pipeline"].shape, "decode", B=8, ctx=3000), {}),
    "small_prefill": lambda: (WL.Workload("pre", WL.LayerShape(H=512, nq=8, nkv=2, d=64, F=1376), "prefill", B=3, seq_tokens=130), {}),
    "prefill_glu_epilogue": lambda: (WL.Workload("glu", WL.LayerShape(H=512, nq=8, nkv=2, d=64, F=3072), "prefill", B=2, seq_tokens=1024), {}),
}


@pytest.mark.parametrize("case", list(CASES))
def test_kernels_stay_inside_their_declared_accesses(B, case):
    wl, _ = CASES[case]()
    weights, io, _ = WL.build(wl, seed=3)
    Lcap = io["kcache"].shape[2]
    if wl.mode == "decode":          # room behind the appended position, so that there is a tail to poison
        pad = torch.zeros(wl.B, wl.shape.nkv, 7, wl.shape.d, dtype=torch.bfloat16)
        io["kcache"] = torch.cat([io["kcache"], pad], dim=2).contiguous()
        io["vcache"] = torch.cat([io["vcache"], pad], dim=2).contiguous()
    a = run_declared(B, wl, weights, io, ws_fill=0xFF, tail_fill=float("nan"))
    b = run_declared(B, wl, weights, io, ws_fill=0xA5, tail_fill=-3.0)
    assert len(a) == len(b) and len(a) > 0
    for (ka, u), (kb, v) in zip(a, b):
        assert ka == kb
        assert torch.equal(u.view(torch.uint8).reshape(-1), v.view(torch.uint8).reshape(-1)), \
            f"declared output (buffer, offset, extent) = {ka} depends on bytes this call did not write first"
