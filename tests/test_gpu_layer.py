"""Whole-layer and pipelined-step parity at small sizes (every boundary tensor is compared),
including the MoE layer with teacher-forced routing and the prefill -> decode hand-over."""
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


def run_layer(B, wl, weights, io, use_table=False):
    """Runs ts_layer_forward; returns dict of boundary tensors (numpy f64) + caches."""
    s = wl.shape
    Lcap = io["kcache"].shape[2]
    T = io["x"].shape[0]
    Bs = io["kcache"].shape[0]
    wd = {k: v.to(DEV) for k, v in weights.items()}
    iod = {k: v.to(DEV) for k, v in io.items()}
    out = torch.empty(T, s.H, dtype=torch.bfloat16, device=DEV)
    desc = B.make_desc(s, Lcap, wl.mode)
    table = None
    if use_table:
        th = torch.empty(Lcap, s.d, dtype=torch.float32)
        B.ts_rope_table(th, Lcap, s.d, s.rope_base)
        table = th.to(DEV)
    nbytes = B.ts_layer_workspace_bytes(desc, T, Bs)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    max_seqlen = int(io["seq_lens"].max()) if wl.mode == "prefill" else 0
    B.ts_layer_forward(desc, B.make_weights(wd, table), B.make_io(iod, out, T, Bs, max_seqlen), ws)
    torch.cuda.synchronize()
    names = O.BOUNDARY_ORDER_MOE if s.E else O.BOUNDARY_ORDER_DENSE
    names = [n for n in names if n != "logits"]
    res = {}
    for i, n in enumerate(names):
        off, nb = B.ts_layer_boundary(desc, T, Bs, i)
        if off is None:
            res[n] = to_np(out)
        else:
            res[n] = to_np(ws[off:off + nb].view(torch.bfloat16))
    if s.E:
        offs = B.ts_layer_moe_buffers(desc, T, Bs)
        k = s.k
        res["logits"] = ws[offs[0]:offs[0] + T * s.E * 4].view(torch.float32).cpu().numpy().reshape(T, s.E)
        res["topk_idx"] = ws[offs[1]:offs[1] + T * k * 4].view(torch.int32).cpu().numpy().reshape(T, k)
        res["topk_w"] = ws[offs[2]:offs[2] + T * k * 4].view(torch.float32).cpu().numpy().reshape(T, k)
        res["counts"] = ws[offs[3]:offs[3] + s.E * 4].view(torch.int32).cpu().numpy()
        res["offsets"] = ws[offs[4]:offs[4] + (s.E + 1) * 4].view(torch.int32).cpu().numpy()
        res["perm"] = ws[offs[5]:offs[5] + T * k * 4].view(torch.int32).cpu().numpy()
    res["kcache"] = to_np(iod["kcache"])
    res["vcache"] = to_np(iod["vcache"])
    return res


def oracle_layer(wl, weights, io, **kw):
    w64 = {k: WL.as_f64(v) for k, v in weights.items()}
    io64 = {k: WL.as_f64(v) for k, v in io.items()}
    r = O.layer_forward(wl.shape, w64, io64, wl.mode, **kw)
    r["kcache"], r["vcache"] = io64["kcache"], io64["vcache"]
    return r


def compare_layer(got, ref, names):
    for n in names:
        assert_close(got[n].reshape(-1), ref[n].reshape(-1), f"boundary {n}")
    assert_close(got["kcache"], ref["kcache"], "kcache")
    assert_close(got["vcache"], ref["vcache"], "vcache")


@pytest.mark.parametrize("use_table", [False, True])
def test_tiny_decode_layer_all_boundaries(B, use_table):
    wl = WL.CONFIGS["tiny"]
    weights, io, _ = WL.build(wl)
    got = run_layer(B, wl, weights, io, use_table)
    ref = oracle_layer(wl, weights, io)
    compare_layer(got, ref, O.BOUNDARY_ORDER_DENSE)


def test_small_ragged_decode_layer_nan_tail(B):
    """Ragged lengths, unused cache tail poisoned with NaN: nothing beyond seq_lens may be read."""
    wl = WL.scaled(WL.CONFIGS["tiny"], B=5)
    weights, io, _ = WL.build(wl, seed=3, ctx_lens=[0, 1, 31, 300, 77], tail_fill=float("nan"))
    got = run_layer(B, wl, weights, io)
    io_o = {k: (torch.nan_to_num(v, nan=0.0) if v.is_floating_point() else v) for k, v in io.items()}
    ref = oracle_layer(wl, weights, io_o)
    for n in O.BOUNDARY_ORDER_DENSE:
        assert_close(got[n].reshape(-1), ref[n].reshape(-1), f"boundary {n}")


def test_mid_decode_layer_gqa8(B):
    """A 70B-like head layout (GQA group 8, d=128) at reduced width."""
    shape = WL.LayerShape(H=1024, nq=16, nkv=2, d=128, F=2816)
    wl = WL.Workload("mid", shape, "decode", B=6)
    weights, io, _ = WL.build(wl, seed=1, ctx_lens=[512, 1500, 33, 2048, 700, 1])
    got = run_layer(B, wl, weights, io, use_table=True)
    ref = oracle_layer(wl, weights, io)
    compare_layer(got, ref, O.BOUNDARY_ORDER_DENSE)


def test_small_prefill_layer_then_decode(B):
    shape = WL.LayerShape(H=512, nq=8, nkv=2, d=64, F=1376)
    wl = WL.Workload("pre", shape, "prefill", B=3, seq_tokens=0)
    gen = torch.Generator().manual_seed(7)
    weights = WL.make_weights(shape, gen)
    seqs = [70, 1, 130]
    io = WL.make_prefill_io(shape, seqs, gen, Lcap=140)
    got = run_layer(B, wl, weights, io)
    ref = oracle_layer(wl, weights, io)
    compare_layer(got, ref, O.BOUNDARY_ORDER_DENSE)
    # decode one more token per sequence over the cache the GPU prefill wrote
    wl_d = WL.Workload("dec", shape, "decode", B=3)
    io_d = {"x": WL.randn_bf16(gen, 3, shape.H), "pos": torch.tensor(seqs, dtype=torch.int32),
            "seq_id": torch.arange(3, dtype=torch.int32), "seq_lens": torch.tensor(seqs, dtype=torch.int32) + 1,
            "kcache": torch.tensor(got["kcache"]).to(torch.bfloat16), "vcache": torch.tensor(got["vcache"]).to(torch.bfloat16)}
    got_d = run_layer(B, wl_d, weights, io_d)
    ref_d = oracle_layer(wl_d, weights, io_d)
    compare_layer(got_d, ref_d, O.BOUNDARY_ORDER_DENSE)


def test_prefill_layer_with_the_activation_in_the_projection_epilogue(B):
    """2048 tokens x F = 3072 is the smallest shape whose gate/up projection takes the 256 x 256 MFMA kernel
    with SwiGLU applied in its epilogue: gate_up and act must both be what the separate kernels produce."""
    shape = WL.LayerShape(H=512, nq=8, nkv=2, d=64, F=3072)
    wl = WL.Workload("glu", shape, "prefill", B=3, seq_tokens=0)
    gen = torch.Generator().manual_seed(13)
    weights = WL.make_weights(shape, gen)
    seqs = [1000, 24, 1024]
    io = WL.make_prefill_io(shape, seqs, gen, Lcap=1024)
    got = run_layer(B, wl, weights, io)
    ref = oracle_layer(wl, weights, io)
    compare_layer(got, ref, O.BOUNDARY_ORDER_DENSE)
    # act is exactly silu(gate) * up of the bf16 gate_up the kernel wrote (fp32 arithmetic, one rounding)
    gu = torch.tensor(got["gate_up"]).reshape(sum(seqs), 2 * shape.F).float()
    g, u = gu[:, :shape.F], gu[:, shape.F:]
    want = (g / (1.0 + torch.exp(-g)) * u).to(torch.bfloat16).double().numpy()
    diff = np.abs(got["act"].reshape(want.shape) - want)
    tol = np.maximum(np.abs(want) * 2.0 ** -7, 1e-30)          # at most one bf16 ulp (exp is the device's fast one)
    assert np.all(diff <= tol)


@pytest.mark.parametrize("E", [8, 17])
def test_small_moe_layer_teacher_forced(B, E):
    """E = 17: more experts than the router kernel takes, so the logits come from the projection kernels with an
    fp32 result, an odd number of columns and K split across workgroups."""
    shape = WL.LayerShape(H=512, nq=8, nkv=2, d=64, F=688, E=E, k=2)
    wl = WL.Workload("moe", shape, "decode", B=48)
    weights, io, _ = WL.build(wl, seed=2, ctx_lens=[100 + 3 * i for i in range(48)])
    got = run_layer(B, wl, weights, io)
    ref_free = oracle_layer(wl, weights, io)
    for n in ("h1", "qkv", "attn", "x2", "h2"):
        assert_close(got[n].reshape(-1), ref_free[n].reshape(-1), f"boundary {n}")
    assert_close(got["logits"], ref_free["logits"], "router logits", max_abs=2e-2, rel_l2=5e-3)
    # routing is exact given the logits the GPU produced (same fp32 values on both sides)
    idx, w, counts, offsets, perm = O.moe_route(got["logits"], shape.k)
    assert np.array_equal(got["topk_idx"], idx)
    assert np.array_equal(got["counts"], counts)
    assert np.array_equal(got["offsets"], offsets)
    assert np.array_equal(got["perm"], perm)
    assert np.allclose(got["topk_w"], w, atol=2e-7)
    # teacher-forced: the oracle layer takes the GPU's routing decision, everything else its own
    ref = oracle_layer(wl, weights, io, forced_route=(idx, w))
    for n in ("gate_up", "act", "y", "out"):
        assert_close(got[n].reshape(-1), ref[n].reshape(-1), f"boundary {n}")
    # and un-forced routing agrees wherever the top-k margin is clear of bf16 noise
    srt = np.sort(ref_free["logits"], axis=1)[:, ::-1]
    clear = (srt[:, shape.k - 1] - srt[:, shape.k]) > 2e-2
    assert np.array_equal(got["topk_idx"][clear], ref_free["topk_idx"][clear])


def _pipeline_case(B, wl, weights, io, n_mb, mask, sizes=None):
    """Runs ts_pipeline_step nine times on the same pipeline object (copy modes, slot geometries, KV delta, slower
    link) and checks every micro-batch bit for bit against ts_layer_forward on that micro-batch alone.
    sizes: sequences per micro-batch (default: equal shares)."""
    s = wl.shape
    Lcap = io["kcache"].shape[2]
    sizes = list(sizes) if sizes is not None else [wl.B // n_mb] * n_mb
    assert len(sizes) == n_mb and sum(sizes) == wl.B
    starts = [sum(sizes[:i]) for i in range(n_mb)]
    nb = B.TS_NB_MOE if s.E else B.TS_NB_DENSE
    wd = {k: v.to(DEV) for k, v in weights.items()}
    desc = B.make_desc(s, Lcap, "decode")
    wts = B.make_weights(wd)
    # reference runs: one ts_layer_forward per micro-batch on private cache copies
    singles, ios_dev, outs = [], [], []
    for i in range(n_mb):
        per = sizes[i]
        sl = slice(starts[i], starts[i] + per)
        iod = {k: (v[sl].clone().to(DEV) if k != "seq_id" else torch.arange(per, dtype=torch.int32, device=DEV))
               for k, v in io.items()}
        out = torch.empty(per, s.H, dtype=torch.bfloat16, device=DEV)
        ws1 = torch.zeros(B.ts_layer_workspace_bytes(desc, per, per), dtype=torch.uint8, device=DEV)
        iod1 = {k: v.clone() for k, v in iod.items()}
        B.ts_layer_forward(desc, wts, B.make_io(iod1, out, per, per), ws1)
        torch.cuda.synchronize()
        rows = []
        for j in range(nb):
            if not (mask >> j) & 1:
                continue
            off, nbytes = B.ts_layer_boundary(desc, per, per, j)
            rows.append(out.view(torch.uint8).reshape(-1).clone() if off is None else ws1[off:off + nbytes].clone())
        singles.append((out.clone(), torch.cat(rows) if rows else torch.zeros(0, dtype=torch.uint8, device=DEV),
                        iod1["kcache"].clone()))
        ios_dev.append(iod)
        outs.append(torch.empty(per, s.H, dtype=torch.bfloat16, device=DEV))
    pmax = max(sizes)
    stride = B.ts_pipeline_slot_stride(desc, pmax, pmax, mask)
    layouts = [B.ts_pipeline_boundary_layout(desc, n, n, mask) for n in sizes]
    staging = torch.zeros(max(stride * n_mb, 16), dtype=torch.uint8, device=DEV)
    host = torch.zeros(max(stride * n_mb, 16), dtype=torch.uint8).pin_memory()
    slot = B.ts_pipeline_workspace_slot_bytes(desc, sizes, sizes)
    assert slot >= max(B.ts_layer_workspace_bytes(desc, n, n) for n in sizes)
    ws = torch.zeros(2 * slot, dtype=torch.uint8, device=DEV)
    ws_odd = torch.zeros(3 * slot, dtype=torch.uint8, device=DEV)
    ws_wide = torch.zeros(n_mb * slot, dtype=torch.uint8, device=DEV)
    pipe = B.ts_pipeline_create(desc, n_mb)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    copy = torch.cuda.Stream()
    delta_stream = torch.cuda.Stream()
    dstride = B.ts_pipeline_kv_delta_stride(desc, pmax)
    assert dstride >= pmax * 2 * s.nkv * s.d * 2 and dstride % 256 == 0
    delta_dev = torch.zeros(dstride * n_mb, dtype=torch.uint8, device=DEV)
    delta_host = torch.zeros(dstride * n_mb, dtype=torch.uint8).pin_memory()
    torch.cuda.synchronize()
    try:
        # later repetitions reuse staging slots and workspace slots; the third coalesces sends at four points of
        # the layer, the fourth at two, the fifth gets a workspace slot per micro-batch (another slot geometry
        # than the step before it, so it waits for all of that step's transfers)
        # the sixth crosses the host link three times per tensor (slower-link emulation): same bytes in the slots;
        # the seventh and eighth run on three workspace slots: a slot's next user then sits on the OTHER compute
        # stream, and nothing but the end-of-micro-batch event orders the two (with no boundary flagged, or only
        # an early one, the sends do not); the ninth goes back to two slots right behind it
        for rep in range(9):
            # the KV delta is replicated in the background from the second repetition on (off again for the
            # three-slot repetitions, where it would order the streams by itself)
            if rep >= 1:
                B.ts_pipeline_set_kv_delta(pipe, delta_stream, delta_dev, delta_host)
                delta_host.zero_()
            if rep in (6, 7):
                B.ts_pipeline_set_kv_delta(pipe, None, None, None)
            caches = [{k: v.clone() for k, v in ios_dev[i].items()} for i in range(n_mb)]
            mbs = [B.make_io(caches[i], outs[i], sizes[i], sizes[i]) for i in range(n_mb)]
            for o in outs:
                o.zero_()
            host.zero_()
            mode = {2: B.TS_PIPE_COPY_COALESCED, 3: B.TS_PIPE_COPY_COALESCED_HALVES,
                    5: B.TS_PIPE_COPY_COALESCED, 7: B.TS_PIPE_COPY_SERIALISED}.get(rep, B.TS_PIPE_COPY_SIDE_STREAM)
            if rep == 5:
                with pytest.raises(B.TesseraError):
                    B.ts_pipeline_set_link_slowdown(pipe, 0)
                B.ts_pipeline_set_link_slowdown(pipe, 3)
            if rep == 6:
                B.ts_pipeline_set_link_slowdown(pipe, 1)
            wbuf = ws_wide if rep == 4 else (ws_odd if rep in (6, 7) else ws)
            torch.cuda.synchronize()
            B.ts_pipeline_step(pipe, wts, mbs, streams, copy, mask, staging, host, wbuf, copy_mode=mode)
            if rep in (6, 7):   # a second step right behind it, no host synchronisation in between
                B.ts_pipeline_step(pipe, wts, mbs, streams, copy, mask, staging, host, wbuf, copy_mode=mode)
            for st in streams + [copy, delta_stream]:
                st.synchronize()
            if rep >= 1 and rep not in (6, 7):
                # slot i = for every token its new K row then its new V row, exactly what the cache holds at its position
                for i in range(n_mb):
                    c = caches[i]
                    idx_s = c["seq_id"].long()
                    idx_p = c["pos"].long()
                    k_new = c["kcache"][idx_s, :, idx_p, :].reshape(sizes[i], -1)
                    v_new = c["vcache"][idx_s, :, idx_p, :].reshape(sizes[i], -1)
                    want = torch.cat([k_new, v_new], dim=1).contiguous().view(torch.uint8).reshape(-1).cpu()
                    got = delta_host[i * dstride:i * dstride + want.numel()]
                    assert torch.equal(got, want), f"micro-batch {i}: KV delta differs from the appended cache rows"
                    assert torch.equal(delta_dev[i * dstride:i * dstride + want.numel()].cpu(), want)
            for i in range(n_mb):
                assert torch.equal(outs[i], singles[i][0]), f"rep {rep} micro-batch {i}: output differs from the single-stream layer"
                assert torch.equal(caches[i]["kcache"], singles[i][2])
                got = host[i * stride:i * stride + layouts[i][-1]]
                assert torch.equal(got, singles[i][1].cpu()), f"rep {rep} micro-batch {i}: pinned-host boundary bytes differ"
    finally:
        B.ts_pipeline_destroy(pipe)
    return singles, layouts


@pytest.mark.parametrize("mask", [~0, 0b10001000, 0b1000, 0])
def test_pipeline_step_matches_single_stream_and_oracle(B, mask):
    wl = WL.scaled(WL.CONFIGS["tiny"], B=8)
    weights, io, lens = WL.build(wl, seed=5, ctx_lens=[128, 64, 1, 300, 17, 200, 5, 90])
    mask &= 0xFF
    singles, layouts = _pipeline_case(B, wl, weights, io, 4, mask)
    # and the shipped bytes are the oracle's boundary tensors within tolerance
    per = 2
    for i in range(4):
        sl = slice(i * per, (i + 1) * per)
        io_i = {k: v[sl] for k, v in io.items()}
        io_i["seq_id"] = torch.arange(per, dtype=torch.int32)
        w64 = {k: WL.as_f64(v) for k, v in weights.items()}
        r = O.layer_forward(wl.shape, w64, {k: WL.as_f64(v) for k, v in io_i.items()}, "decode")
        ref = O.boundary_stream(r, moe=False, mask=mask)
        got = singles[i][1].view(torch.bfloat16)
        assert got.numel() == ref.size
        if ref.size:
            assert_close(got, ref, f"micro-batch {i} boundary stream")


def test_pipeline_step_micro_batches_of_different_sizes(B):
    """Micro-batches of 5, 1, 4 and 2 sequences: each lays its workspace slot out with its own plan, the slot is the
    largest of them, staging slots use the stride of the largest."""
    shape = WL.LayerShape(H=512, nq=8, nkv=2, d=64, F=1376)
    wl = WL.Workload("ragged_mb", shape, "decode", B=12)
    weights, io, _ = WL.build(wl, seed=9, ctx_lens=[40, 3000, 17, 1, 260, 2500, 64, 5000, 9, 130, 77, 300])
    _pipeline_case(B, wl, weights, io, 4, 0xFF, sizes=[5, 1, 4, 2])
    # a workspace of two slots sized for the largest micro-batch alone is refused when another one needs more
    desc = B.make_desc(shape, io["kcache"].shape[2], "decode")
    need = B.ts_pipeline_workspace_slot_bytes(desc, [5, 1, 4, 2], [5, 1, 4, 2])
    assert need >= max(B.ts_layer_workspace_bytes(desc, n, n) for n in (5, 1, 4, 2))


@pytest.mark.parametrize("mask", [0xFF, 0b00100100])
def test_pipeline_step_over_prompts(B, mask):
    """Prefill through the pipelined step (the paper pipelines whole requests, prompt phase included): micro-batches
    are packed prompts of different lengths, each with a fresh cache.  Outputs, written caches, shipped boundary
    bytes and the KV delta (here every prompt token's K and V row) are bit-identical to ts_layer_forward on the
    micro-batch alone; the shipped bytes match the oracle's boundary tensors within tolerance."""
    shape = WL.LayerShape(H=512, nq=8, nkv=2, d=64, F=1376)
    prompts = [[70, 33], [128], [5, 64, 17], [1, 200]]
    Lcap = 256
    gen = torch.Generator().manual_seed(21)
    weights = WL.make_weights(shape, gen)
    wd = {k: v.to(DEV) for k, v in weights.items()}
    desc = B.make_desc(shape, Lcap, "prefill")
    wts = B.make_weights(wd)
    nb = B.TS_NB_DENSE
    n_mb = len(prompts)
    ios, singles, Ts, Bs = [], [], [], []
    for seqs in prompts:
        io = WL.make_prefill_io(shape, seqs, gen, Lcap=Lcap)
        T, nseq = sum(seqs), len(seqs)
        iod = {k: v.to(DEV) for k, v in io.items()}
        out = torch.empty(T, shape.H, dtype=torch.bfloat16, device=DEV)
        ws1 = torch.zeros(B.ts_layer_workspace_bytes(desc, T, nseq), dtype=torch.uint8, device=DEV)
        iod1 = {k: v.clone() for k, v in iod.items()}
        B.ts_layer_forward(desc, wts, B.make_io(iod1, out, T, nseq, max(seqs)), ws1)
        torch.cuda.synchronize()
        rows = []
        for j in range(nb):
            if (mask >> j) & 1:
                off, nbytes = B.ts_layer_boundary(desc, T, nseq, j)
                rows.append(out.view(torch.uint8).reshape(-1).clone() if off is None else ws1[off:off + nbytes].clone())
        singles.append((out.clone(), torch.cat(rows), iod1["kcache"].clone(), iod1["vcache"].clone()))
        ios.append((io, iod))
        Ts.append(T)
        Bs.append(nseq)
    Tmax, Bmax = max(Ts), max(Bs)
    stride = B.ts_pipeline_slot_stride(desc, Tmax, Bmax, mask)
    layouts = [B.ts_pipeline_boundary_layout(desc, Ts[i], Bs[i], mask) for i in range(n_mb)]
    staging = torch.zeros(stride * n_mb, dtype=torch.uint8, device=DEV)
    host = torch.zeros(stride * n_mb, dtype=torch.uint8).pin_memory()
    slot = B.ts_pipeline_workspace_slot_bytes(desc, Ts, Bs)
    dstride = B.ts_pipeline_kv_delta_stride(desc, Tmax)
    assert dstride >= Tmax * 2 * shape.nkv * shape.d * 2
    delta_dev = torch.zeros(dstride * n_mb, dtype=torch.uint8, device=DEV)
    delta_host = torch.zeros(dstride * n_mb, dtype=torch.uint8).pin_memory()
    pipe = B.ts_pipeline_create(desc, n_mb)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    copy, delta_stream = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    try:
        B.ts_pipeline_set_kv_delta(pipe, delta_stream, delta_dev, delta_host)
        for rep, (mode, nslot) in enumerate([(B.TS_PIPE_COPY_SIDE_STREAM, 2), (B.TS_PIPE_COPY_COALESCED, 3),
                                             (B.TS_PIPE_COPY_COALESCED_HALVES, 2), (B.TS_PIPE_COPY_SERIALISED, n_mb)]):
            ws = torch.zeros(nslot * slot, dtype=torch.uint8, device=DEV)
            caches = [{k: v.clone() for k, v in ios[i][1].items()} for i in range(n_mb)]
            outs = [torch.zeros(Ts[i], shape.H, dtype=torch.bfloat16, device=DEV) for i in range(n_mb)]
            mbs = [B.make_io(caches[i], outs[i], Ts[i], Bs[i], max(prompts[i])) for i in range(n_mb)]
            host.zero_()
            delta_host.zero_()
            torch.cuda.synchronize()
            B.ts_pipeline_step(pipe, wts, mbs, streams, copy, mask, staging, host, ws, copy_mode=mode)
            for st in streams + [copy, delta_stream]:
                st.synchronize()
            for i in range(n_mb):
                assert torch.equal(outs[i], singles[i][0]), f"rep {rep} micro-batch {i}: output"
                assert torch.equal(caches[i]["kcache"], singles[i][2]) and torch.equal(caches[i]["vcache"], singles[i][3])
                got = host[i * stride:i * stride + layouts[i][-1]]
                assert torch.equal(got, singles[i][1].cpu()), f"rep {rep} micro-batch {i}: pinned-host boundary bytes"
                c = caches[i]
                k_new = c["kcache"][c["seq_id"].long(), :, c["pos"].long(), :].reshape(Ts[i], -1)
                v_new = c["vcache"][c["seq_id"].long(), :, c["pos"].long(), :].reshape(Ts[i], -1)
                want = torch.cat([k_new, v_new], dim=1).contiguous().view(torch.uint8).reshape(-1).cpu()
                assert torch.equal(delta_host[i * dstride:i * dstride + want.numel()], want), f"rep {rep} micro-batch {i}: KV delta"
    finally:
        B.ts_pipeline_destroy(pipe)
    w64 = {k: WL.as_f64(v) for k, v in weights.items()}
    for i in range(n_mb):
        r = O.layer_forward(shape, w64, {k: WL.as_f64(v) for k, v in ios[i][0].items()}, "prefill")
        ref = O.boundary_stream(r, moe=False, mask=mask)
        got = singles[i][1].view(torch.bfloat16)
        assert got.numel() == ref.size
        assert_close(got, ref, f"micro-batch {i} boundary stream")


@pytest.mark.parametrize("mask", [0x1FF, 0b010100000, 0])
def test_pipeline_step_over_a_moe_layer(B, mask):
    """The MoE layer has nine kernel boundaries (the expert outputs before the weighted combine are one of them);
    all copy modes, bit-identical to the single-stream layer, shipped bytes against the oracle with the routing
    decision of the GPU teacher-forced."""
    shape = WL.LayerShape(H=256, nq=4, nkv=2, d=64, F=688, E=4, k=2)
    wl = WL.Workload("moe_pipe", shape, "decode", B=12)
    weights, io, _ = WL.build(wl, seed=17, ctx_lens=[128, 64, 1, 300, 17, 200, 5, 90, 33, 150, 2, 260])
    singles, layouts = _pipeline_case(B, wl, weights, io, 4, mask)
    per = 3
    w64 = {k: WL.as_f64(v) for k, v in weights.items()}
    names = [n for n in O.BOUNDARY_ORDER_MOE if n != "logits"]
    for i in range(4):
        sl = slice(i * per, (i + 1) * per)
        io_i = {k: v[sl] for k, v in io.items()}
        io_i["seq_id"] = torch.arange(per, dtype=torch.int32)
        got = singles[i][1].view(torch.bfloat16)
        r = O.layer_forward(shape, w64, {k: WL.as_f64(v) for k, v in io_i.items()}, "decode")
        # attention half: free-running oracle; expert half: routing forced to what the oracle decides from its own
        # logits unless the GPU's h2 tips a near-tie (then the shipped tensors are compared per selected expert
        # through the teacher-forced oracle of the small-MoE test above; here margins are asserted instead)
        srt = np.sort(r["logits"], axis=1)[:, ::-1]
        assert np.all(srt[:, shape.k - 1] - srt[:, shape.k] > 1e-3), "seeded router margins are clear at this size"
        parts = [np.asarray(r[n], np.float64).reshape(-1) for j, n in enumerate(names) if (mask >> j) & 1]
        ref = np.concatenate(parts) if parts else np.zeros(0)
        assert got.numel() == ref.size
        if ref.size:
            assert_close(got, ref, f"MoE micro-batch {i} boundary stream")


def test_small_layer_long_contexts_merge_inside_the_attention_launch(B):
    """Sequences of five, three, two and one chunks in one call: the layer takes the attention path that
    combines the chunks in the same launch (last chunk to arrive), and must run it twice in a row with the
    same workspace (the arrival counters are re-armed by the kernel and zeroed by the first norm)."""
    wl = WL.scaled(WL.CONFIGS["tiny"], B=4)
    weights, io, lens = WL.build(wl, seed=21, ctx_lens=[9000, 4097, 2300, 100])
    ref = oracle_layer(wl, weights, io)
    for rep in range(2):
        got = run_layer(B, wl, weights, io)
        compare_layer(got, ref, O.BOUNDARY_ORDER_DENSE)


@pytest.mark.parametrize("moe,lens", [(False, [70, 1, 128, 33, 5, 90]), (True, [70, 1, 128, 33, 5, 90]),
                                      (False, [9000, 1, 4500, 33, 8191, 640])])
def test_layer_forward_replays_from_a_hip_graph(B, moe, lens):
    """The layer enqueues kernels only (no allocation, no memset, no host synchronisation), so it can be
    captured once and replayed.  Every replay is checked against the eager result, with eager work and
    synchronisations between the replays.  The long lengths take the balanced form of the decode attention,
    whose arrival counters the layer's first kernel clears on every replay (the workspace is left as the
    previous replay left it on the odd ones)."""
    shape = WL.LayerShape(H=256, nq=4, nkv=2, d=64, F=688, E=4 if moe else 0, k=2 if moe else 0)
    wl = WL.Workload("graph", shape, "decode", B=6, ctx=128)
    weights, io, _ = WL.build(wl, seed=11, ctx_lens=lens)
    s = wl.shape
    Lcap = io["kcache"].shape[2]
    T = Bs = wl.B
    wd = {k: v.to(DEV) for k, v in weights.items()}
    desc = B.make_desc(s, Lcap, "decode")
    wts = B.make_weights(wd)
    nbytes = B.ts_layer_workspace_bytes(desc, T, Bs)

    def fresh():
        iod = {k: v.clone().to(DEV) for k, v in io.items()}
        return iod, torch.zeros(T, s.H, dtype=torch.bfloat16, device=DEV), torch.zeros(nbytes, dtype=torch.uint8, device=DEV)

    iod_e, out_e, ws_e = fresh()
    B.ts_layer_forward(desc, wts, B.make_io(iod_e, out_e, T, Bs), ws_e)
    torch.cuda.synchronize()
    iod_g, out_g, ws_g = fresh()
    io_g = B.make_io(iod_g, out_g, T, Bs)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        B.ts_layer_forward(desc, wts, io_g, ws_g)
    torch.cuda.synchronize()
    for rep in range(3):
        out_g.zero_()
        if rep % 2 == 0:
            ws_g.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), f"replay {rep}: output differs from the eager layer"
        assert torch.equal(iod_g["kcache"], iod_e["kcache"]) and torch.equal(iod_g["vcache"], iod_e["vcache"])
        # eager work on other buffers between the replays
        iod_x, out_x, ws_x = fresh()
        B.ts_layer_forward(desc, wts, B.make_io(iod_x, out_x, T, Bs), ws_x)
        torch.cuda.synchronize()
        assert torch.equal(out_x, out_e)
