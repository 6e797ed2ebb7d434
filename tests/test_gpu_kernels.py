"""Per-kernel parity: HIP kernels (through the C ABI) vs the fp64 oracle, element by element,
on seeded inputs whose sizes span several tiles and ragged tails, plus the edge cases."""
import math

import numpy as np
import pytest
import torch

import workloads as WL
from oracle import decoder_layer as O
from parity import assert_close, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2604_10180_amd import binding
    return binding


DEV = "cuda:0"


def gen(seed):
    return torch.Generator().manual_seed(seed)


def dev(t):
    return t.to(DEV)


def ws_bytes(n):
    return torch.empty(max(n, 16), dtype=torch.uint8, device=DEV)


# ------------------------------------------------------------------ RMSNorm
@pytest.mark.parametrize("T,H", [(3, 256), (64, 4096), (17, 8192), (5, 32768), (1, 8)])
def test_rmsnorm(B, T, H):
    g = gen(T * 7 + H)
    x = WL.randn_bf16(g, T, H)
    gamma = WL.randn_bf16(g, H, std=0.02, mean=1.0)
    y = torch.empty(T, H, dtype=torch.bfloat16, device=DEV)
    B.ts_rmsnorm(dev(x), dev(gamma), y, T, H, 1e-5)
    assert_close(y, O.rmsnorm(WL.as_f64(x), WL.as_f64(gamma), 1e-5), f"rmsnorm {T}x{H}")


def test_rmsnorm_in_place_and_unit_rms(B):
    g = gen(5)
    x = WL.randn_bf16(g, 9, 1024, std=3.0)
    ones = torch.ones(1024, dtype=torch.bfloat16)
    xd = dev(x).clone()
    B.ts_rmsnorm(xd, dev(ones), xd, 9, 1024, 0.0)
    y = to_np(xd)
    assert np.allclose(np.sqrt((y * y).mean(axis=1)), 1.0, atol=3e-3)


# ------------------------------------------------------------------ SwiGLU
@pytest.mark.parametrize("T,F", [(2, 688), (64, 14336), (33, 1000)])
def test_swiglu(B, T, F):
    gu = WL.randn_bf16(gen(F), T, 2 * F, std=1.5)
    out = torch.empty(T, F, dtype=torch.bfloat16, device=DEV)
    B.ts_swiglu(dev(gu), out, T, F)
    assert_close(out, O.swiglu(WL.as_f64(gu)), f"swiglu {T}x{F}")


# ------------------------------------------------------------------ RoPE + KV append
@pytest.mark.parametrize("d,nq,nkv,use_table", [(64, 4, 2, True), (128, 32, 8, True), (128, 64, 8, False), (64, 4, 2, False)])
def test_rope_and_append(B, d, nq, nkv, use_table):
    g = gen(d + nq)
    T, Bc, Lcap = 6, 3, 40000 if d == 128 else 300
    pos = torch.tensor([0, 1, 17, 255, Lcap - 1, 5], dtype=torch.int32)
    seq = torch.tensor([0, 1, 2, 0, 1, 2], dtype=torch.int32)
    nqkv = (nq + 2 * nkv) * d
    qkv = WL.randn_bf16(g, T, nqkv)
    kc = torch.zeros(Bc, nkv, Lcap, d, dtype=torch.bfloat16)
    kc[:] = 7.0
    vc = kc.clone()
    table = None
    if use_table:
        th = torch.empty(Lcap, d, dtype=torch.float32)
        B.ts_rope_table(th, Lcap, d, 10000.0)
        table = dev(th)
        # the table itself: cos | sin of pos * base^(-2i/d), checked against a direct fp64 evaluation
        i = np.arange(d // 2)
        ang = np.arange(Lcap)[:, None] * (10000.0 ** (-2.0 * i / d))[None, :]
        assert np.allclose(th[:, : d // 2].numpy(), np.cos(ang), atol=1e-6)
        assert np.allclose(th[:, d // 2:].numpy(), np.sin(ang), atol=1e-6)
    qd, kcd, vcd = dev(qkv).clone(), dev(kc), dev(vc)
    B.ts_rope(qd, qd[:, nq * d:], qd[:, (nq + nkv) * d:], nqkv, nqkv, dev(pos), dev(seq), table,
              Lcap if use_table else 0, kcd, vcd, T, nq, nkv, d, Lcap, 10000.0)
    q64 = WL.as_f64(qkv)
    qr = O.rope(q64[:, : nq * d].reshape(T, nq, d), pos.numpy(), 10000.0)
    kr = O.rope(q64[:, nq * d:(nq + nkv) * d].reshape(T, nkv, d), pos.numpy(), 10000.0)
    vr = q64[:, (nq + nkv) * d:].reshape(T, nkv, d)
    got = to_np(qd)
    assert_close(got[:, : nq * d], qr.reshape(T, -1), "rope q")
    assert_close(got[:, nq * d:(nq + nkv) * d], kr.reshape(T, -1), "rope k")
    assert np.array_equal(got[:, (nq + nkv) * d:], vr.reshape(T, -1)), "v must be untouched"
    kref, vref = WL.as_f64(kc), WL.as_f64(vc)
    O.kv_append(kref, vref, kr, vr, seq.numpy(), pos.numpy())
    kgot, vgot = to_np(kcd), to_np(vcd)
    assert_close(kgot, kref, "k cache after append")
    assert np.array_equal(vgot, vref), "v cache rows are plain copies"
    # the appended k rows are bit-identical to the rotated k the kernel left in place
    for t in range(T):
        assert np.array_equal(kgot[seq[t], :, pos[t], :].reshape(-1), got[t, nq * d:(nq + nkv) * d])


# ------------------------------------------------------------------ GEMM
GEMM_SHAPES = [
    (2, 512, 256), (2, 256, 688), (2, 1376, 256),          # tiny layer, K tail 688 = 5*128 + 48
    (64, 6144, 4096), (64, 4096, 14336), (8, 10240, 8192),  # decode shapes (split-K)
    (100, 1376, 256), (17, 66, 72), (128, 130, 136),        # ragged M/N/K on the skinny kernel, N % 4 != 0
    (80, 320, 264), (96, 4096, 512), (256, 8, 4096),        # 96-row tile; tiny N loops over row blocks
    (130, 320, 264), (300, 1002, 520), (1024, 2048, 1024),  # tiled kernel with tails
    (256, 6144, 4096), (200, 1002, 1544),                   # 128 x 128 tiles split along K (reduce kernel), with tails
    (4096, 4096, 128), (3900, 4104, 192), (3585, 3592, 64),  # 256 x 256 direct-to-LDS kernel: even/odd K steps, ragged M and N
    (8, 8200, 4096), (33, 28674, 520), (64, 28672, 1024),   # seven- and eight-wave streaming workgroups: N tails, K tail, no split
    (32, 4104, 1160), (16, 2056, 136), (24, 130, 8),        # weights staged through LDS (up to 32 rows): N and K tails, K < one chunk row
]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("with_res", [False, True])
def test_gemm(B, M, N, K, with_res):
    g = gen(M + N + K)
    A = WL.randn_bf16(g, M, K)
    W = WL.randn_bf16(g, N, K, std=0.02)
    R = WL.randn_bf16(g, M, N) if with_res else None
    Cd = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    ws = ws_bytes(B.ts_gemm_workspace_bytes(M, N, K))
    B.ts_gemm_bf16(dev(A), dev(W), None if R is None else dev(R), Cd, M, N, K, ws)
    ref = O.gemm(WL.as_f64(A), WL.as_f64(W), None if R is None else WL.as_f64(R))
    assert_close(Cd, ref, f"gemm {M}x{N}x{K} res={with_res}")


def test_gemm_seeded_random_shapes(B):
    """Sixty seeded shapes across the dispatch rules (row tiles, seven/eight-wave workgroups, split K, tails in
    every dimension): none may fall between two kernels' assumptions."""
    rng = np.random.default_rng(2024)
    for case in range(60):
        M = int(rng.choice([1, 3, 8, 16, 17, 31, 33, 64, 65, 100, 128, 129, 200]))
        N = int(rng.integers(1, 1600)) * 2
        K = int(rng.integers(1, 700)) * 8
        if case % 5 == 0:
            N, K = int(rng.choice([4096, 6144, 10240, 28672])), int(rng.choice([512, 1024, 2048]))
        g = gen(1000 + case)
        A = WL.randn_bf16(g, M, K)
        W = WL.randn_bf16(g, N, K, std=0.05)
        R = WL.randn_bf16(g, M, N) if case % 2 else None
        Cd = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
        ws = ws_bytes(B.ts_gemm_workspace_bytes(M, N, K))
        B.ts_gemm_bf16(dev(A), dev(W), None if R is None else dev(R), Cd, M, N, K, ws)
        ref = O.gemm(WL.as_f64(A), WL.as_f64(W), None if R is None else WL.as_f64(R))
        assert_close(Cd, ref, f"case {case}: M={M} N={N} K={K} residual={R is not None}")


@pytest.mark.parametrize("M,N,K", [(256, 8, 4096), (5, 8, 256), (200, 64, 512)])
def test_gemm_f32out(B, M, N, K):
    g = gen(M * N)
    A = WL.randn_bf16(g, M, K)
    W = WL.randn_bf16(g, N, K, std=0.02)
    Cd = torch.empty(M, N, dtype=torch.float32, device=DEV)
    ws = ws_bytes(B.ts_gemm_workspace_bytes(M, N, K))
    B.ts_gemm_bf16_f32out(dev(A), dev(W), Cd, M, N, K, ws)
    ref = O.gemm(WL.as_f64(A), WL.as_f64(W))
    assert_close(Cd, ref, f"gemm f32 {M}x{N}x{K}", max_abs=2e-4, rel_l2=1e-5)


def test_gemm_identity_and_residual_alias(B):
    K = 256
    A = WL.randn_bf16(gen(1), 33, K)
    eye = torch.eye(K, dtype=torch.bfloat16)
    Cd = dev(A).clone()
    ws = ws_bytes(B.ts_gemm_workspace_bytes(33, K, K))
    B.ts_gemm_bf16(dev(A), dev(eye), Cd, Cd, 33, K, K, ws)        # C aliases residual: C = A + A
    assert np.array_equal(to_np(Cd), 2 * WL.as_f64(A))


# ------------------------------------------------------------------ decode attention
DECODE_CASES = [
    (4, 2, 64, [129, 129]),
    (32, 8, 128, [1, 31, 257, 1000, 2049]),
    (64, 8, 128, [700, 33, 4096]),
    (8, 8, 128, [513, 64]),
    (16, 1, 64, [300]),
    (16, 2, 128, [9000, 300, 4097]),     # up to five chunks per sequence: partials + merge kernel
    (8, 1, 128, [140001]),               # one long sequence: 68 chunks, offsets beyond 2^24 elements
]


@pytest.mark.parametrize("nq,nkv,d,lens", DECODE_CASES)
def test_attention_decode(B, nq, nkv, d, lens):
    g = gen(nq + d + len(lens))
    Bs, Lcap = len(lens), max(lens) + 3
    q = WL.randn_bf16(g, Bs, nq, d)
    kc = torch.full((Bs, nkv, Lcap, d), float("nan"), dtype=torch.bfloat16)
    vc = kc.clone()
    for b, L in enumerate(lens):
        kc[b, :, :L] = WL.randn_bf16(g, nkv, L, d)
        vc[b, :, :L] = WL.randn_bf16(g, nkv, L, d)
    sl = torch.tensor(lens, dtype=torch.int32)
    out = torch.empty(Bs, nq, d, dtype=torch.bfloat16, device=DEV)
    ws = ws_bytes(B.ts_attention_decode_workspace_bytes(Bs, nq, nkv, d, Lcap))
    scale = 1 / math.sqrt(d)
    B.ts_attention_decode(dev(q), dev(kc), dev(vc), dev(sl), out, Bs, nq, nkv, d, Lcap, scale, ws)
    ref = O.attention_decode(WL.as_f64(q), WL.as_f32(kc), WL.as_f32(vc), lens, scale)
    assert_close(out, ref, f"decode attention nq={nq} nkv={nkv} d={d} lens={lens}")


def test_attention_decode_seeded_random(B):
    """Twenty seeded cases over head layouts (GQA group 1..16, d 64/128) and length mixes that include empty
    sequences, one key, block and chunk boundaries."""
    rng = np.random.default_rng(77)
    special = [0, 1, 31, 32, 33, 2047, 2048, 2049, 4096, 4225]
    for case in range(20):
        d = int(rng.choice([64, 128]))
        nkv = int(rng.choice([1, 2, 4, 8]))
        g_ = int(rng.choice([1, 2, 4, 8, 16]))
        nq = nkv * g_
        Bs = int(rng.integers(1, 7))
        lens = [int(rng.choice(special)) if rng.random() < 0.5 else int(rng.integers(0, 5000)) for _ in range(Bs)]
        Lcap = max(max(lens), 1) + int(rng.integers(0, 40))
        g = gen(5000 + case)
        q = WL.randn_bf16(g, Bs, nq, d)
        kc = WL.randn_bf16(g, Bs, nkv, Lcap, d)
        vc = WL.randn_bf16(g, Bs, nkv, Lcap, d)
        sl = torch.tensor(lens, dtype=torch.int32)
        out = torch.full((Bs, nq, d), 9.0, dtype=torch.bfloat16, device=DEV)
        ws = ws_bytes(B.ts_attention_decode_workspace_bytes(Bs, nq, nkv, d, Lcap))
        scale = 1 / math.sqrt(d)
        B.ts_attention_decode(dev(q), dev(kc), dev(vc), dev(sl), out, Bs, nq, nkv, d, Lcap, scale, ws)
        ref = O.attention_decode(WL.as_f64(q), WL.as_f32(kc), WL.as_f32(vc), lens, scale)
        assert_close(out, ref, f"case {case}: nq={nq} nkv={nkv} d={d} lens={lens} Lcap={Lcap}")


def test_attention_decode_long_caches_seeded_random(B):
    """Caches long enough for the balanced split (the keys of all (sequence, kv head) pairs cut into equal
    ranges, one per workgroup): length mixes with empty sequences, one key, granule boundaries, full caches, one
    long sequence among short ones, short sequences in a long cache; each case is run twice on the same
    workspace with the sequences in reverse order the second time (the arrival counters must be back at zero)."""
    rng = np.random.default_rng(99)
    for case in range(10):
        d = int(rng.choice([64, 128]))
        nkv = int(rng.choice([1, 2, 4]))
        g_ = int(rng.choice([1, 4, 8, 16]))
        nq = nkv * g_
        Bs = int(rng.integers(1, 11))
        Lcap = int(rng.choice([8200, 12345, 20000]))
        special = [0, 1, 127, 128, 129, 4096, Lcap - 1, Lcap]
        kind = case % 4
        if kind == 0:
            lens = [int(rng.integers(0, Lcap + 1)) for _ in range(Bs)]
        elif kind == 1:
            lens = [int(rng.choice(special)) for _ in range(Bs)]
        elif kind == 2:
            lens = [int(rng.integers(0, 200)) for _ in range(Bs)]
            lens[int(rng.integers(0, Bs))] = Lcap
        else:
            lens = [int(rng.integers(1, 600)) for _ in range(Bs)]
        g = gen(7000 + case)
        q = WL.randn_bf16(g, Bs, nq, d)
        kc = WL.randn_bf16(g, Bs, nkv, Lcap, d)
        vc = WL.randn_bf16(g, Bs, nkv, Lcap, d)
        ws = ws_bytes(B.ts_attention_decode_workspace_bytes(Bs, nq, nkv, d, Lcap))
        scale = 1 / math.sqrt(d)
        qd, kd, vd = dev(q), dev(kc), dev(vc)
        for rnd in range(2):
            order = list(range(Bs)) if rnd == 0 else list(range(Bs))[::-1]
            ls = [lens[i] for i in order]
            sl = torch.tensor(ls, dtype=torch.int32)
            out = torch.full((Bs, nq, d), 9.0, dtype=torch.bfloat16, device=DEV)
            # (the lengths are permuted, the caches are not: sequence b simply attends over another prefix)
            B.ts_attention_decode(qd, kd, vd, dev(sl), out, Bs, nq, nkv, d, Lcap, scale, ws)
            ref = O.attention_decode(WL.as_f64(q), WL.as_f32(kc), WL.as_f32(vc), ls, scale)
            assert_close(out, ref, f"case {case} round {rnd}: nq={nq} nkv={nkv} d={d} lens={ls} Lcap={Lcap}")
            for b, L in enumerate(ls):
                if L == 0:
                    assert torch.all(out[b] == 0), "empty sequence gives a zero row"


def test_attention_decode_degenerate(B):
    g = gen(3)
    nq, nkv, d, Lcap = 8, 2, 128, 64
    q = WL.randn_bf16(g, 3, nq, d)
    kc = WL.randn_bf16(g, 3, nkv, Lcap, d)
    vc = WL.randn_bf16(g, 3, nkv, Lcap, d)
    kc[2] = kc[2, :, :1]                      # identical keys -> uniform weights -> mean of V
    sl = torch.tensor([0, 1, 64], dtype=torch.int32)
    out = torch.full((3, nq, d), 5.0, dtype=torch.bfloat16, device=DEV)
    ws = ws_bytes(B.ts_attention_decode_workspace_bytes(3, nq, nkv, d, Lcap))
    B.ts_attention_decode(dev(q), dev(kc), dev(vc), dev(sl), out, 3, nq, nkv, d, Lcap, 0.1, ws)
    got = to_np(out)
    assert np.all(got[0] == 0.0), "empty sequence gives a zero row"
    v = WL.as_f64(vc)
    for h in range(nq):
        assert np.array_equal(got[1, h], v[1, h // 4, 0]), "single key returns that V row exactly"
    assert_close(got[2], np.repeat(v[2].mean(axis=1), 4, axis=0), "uniform attention = mean of V")


# ------------------------------------------------------------------ prefill attention
@pytest.mark.parametrize("nq,nkv,d,seqs,causal", [
    (4, 2, 64, [1, 63, 64, 65, 200], True),
    (8, 2, 128, [130, 31, 257], True),
    (4, 4, 128, [100, 70], False),
    (16, 2, 128, [300, 129], True),      # GQA group 8: eight heads per workgroup, 32-query blocks
    (6, 2, 64, [97, 260], True),         # group 3: one head per workgroup, 256-query blocks
    (8, 8, 64, [513], False),            # no GQA, non-causal, ragged tail block
    (32, 8, 128, [1000, 24], True),      # the 8B head layout over several query and key blocks
])
def test_attention_prefill(B, nq, nkv, d, seqs, causal):
    g = gen(sum(seqs) + d)
    T = sum(seqs)
    nqkv = (nq + 2 * nkv) * d
    qkv = WL.randn_bf16(g, T, nqkv)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(seqs)]), dtype=torch.int32)
    out = torch.empty(T, nq, d, dtype=torch.bfloat16, device=DEV)
    qd = dev(qkv)
    scale = 1 / math.sqrt(d)
    B.ts_attention_prefill(qd, qd[:, nq * d:], qd[:, (nq + nkv) * d:], nqkv, nqkv, dev(cu), out, len(seqs), T,
                           max(seqs), nq, nkv, d, scale, causal)
    x = WL.as_f64(qkv)
    ref = O.attention_prefill(x[:, : nq * d].reshape(T, nq, d), x[:, nq * d:(nq + nkv) * d].reshape(T, nkv, d),
                              x[:, (nq + nkv) * d:].reshape(T, nkv, d), cu.numpy(), scale, causal)
    assert_close(out, ref, f"prefill attention seqs={seqs} causal={causal}")


def test_attention_prefill_seeded_random(B):
    """Twelve seeded cases: GQA groups 1..8, d 64/128, causal or not, sequence lengths around the 32-query and
    64-key block edges, empty sequences between others."""
    rng = np.random.default_rng(99)
    edges = [0, 1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257]
    for case in range(12):
        d = int(rng.choice([64, 128]))
        nkv = int(rng.choice([1, 2, 4]))
        nq = nkv * int(rng.choice([1, 2, 3, 4, 6, 8]))
        seqs = [int(rng.choice(edges)) if rng.random() < 0.6 else int(rng.integers(1, 600)) for _ in range(int(rng.integers(1, 5)))]
        if sum(seqs) == 0:
            seqs.append(70)
        causal = bool(case % 3)
        g = gen(7000 + case)
        T = sum(seqs)
        nqkv = (nq + 2 * nkv) * d
        qkv = WL.randn_bf16(g, T, nqkv)
        cu = torch.tensor(np.concatenate([[0], np.cumsum(seqs)]), dtype=torch.int32)
        out = torch.full((T, nq, d), 9.0, dtype=torch.bfloat16, device=DEV)
        qd = dev(qkv)
        scale = 1 / math.sqrt(d)
        B.ts_attention_prefill(qd, qd[:, nq * d:], qd[:, (nq + nkv) * d:], nqkv, nqkv, dev(cu), out, len(seqs), T,
                               max(seqs), nq, nkv, d, scale, causal)
        x = WL.as_f64(qkv)
        ref = O.attention_prefill(x[:, : nq * d].reshape(T, nq, d), x[:, nq * d:(nq + nkv) * d].reshape(T, nkv, d),
                                  x[:, (nq + nkv) * d:].reshape(T, nkv, d), cu.numpy(), scale, causal)
        assert_close(out, ref, f"case {case}: nq={nq} nkv={nkv} d={d} seqs={seqs} causal={causal}")


# ------------------------------------------------------------------ MoE
def test_moe_route_exact(B):
    g = gen(11)
    T, E, k = 300, 8, 2
    lg = torch.randn(T, E, generator=g, dtype=torch.float32)
    lg[0] = torch.tensor([1., 3., 3., 0., 3., -1., 0., 0.])       # ties -> lower index first
    lg[1] = 5.0
    lg[2, 3] = lg[2, 6] = 9.0
    outs = [torch.empty(T, k, dtype=torch.int32, device=DEV), torch.empty(T, k, dtype=torch.float32, device=DEV),
            torch.empty(E, dtype=torch.int32, device=DEV), torch.empty(E + 1, dtype=torch.int32, device=DEV),
            torch.empty(T * k, dtype=torch.int32, device=DEV)]
    B.ts_moe_route(dev(lg), T, E, k, *outs)
    idx, w, counts, offsets, perm = O.moe_route(lg.numpy(), k)
    assert np.array_equal(outs[0].cpu().numpy(), idx)
    assert np.array_equal(outs[2].cpu().numpy(), counts)
    assert np.array_equal(outs[3].cpu().numpy(), offsets)
    assert np.array_equal(outs[4].cpu().numpy(), perm)
    assert np.allclose(outs[1].cpu().numpy(), w, atol=2e-7)
    assert np.allclose(outs[1].cpu().numpy().sum(axis=1), 1.0, atol=1e-6)


@pytest.mark.parametrize("T,E,k", [(1, 4, 1), (7, 64, 8), (2000, 16, 4)])
def test_moe_route_shapes(B, T, E, k):
    lg = torch.randn(T, E, generator=gen(T + E), dtype=torch.float32)
    outs = [torch.empty(T, k, dtype=torch.int32, device=DEV), torch.empty(T, k, dtype=torch.float32, device=DEV),
            torch.empty(E, dtype=torch.int32, device=DEV), torch.empty(E + 1, dtype=torch.int32, device=DEV),
            torch.empty(T * k, dtype=torch.int32, device=DEV)]
    B.ts_moe_route(dev(lg), T, E, k, *outs)
    idx, w, counts, offsets, perm = O.moe_route(lg.numpy(), k)
    for got, ref in zip((outs[0], outs[2], outs[3], outs[4]), (idx, counts, offsets, perm)):
        assert np.array_equal(got.cpu().numpy(), ref)
    assert np.allclose(outs[1].cpu().numpy(), w, atol=2e-7)


@pytest.mark.parametrize("T,E,k,H,N", [(40, 4, 2, 256, 688), (256, 8, 2, 512, 1024), (9, 8, 2, 128, 64), (600, 3, 1, 64, 130),
                                       (256, 8, 2, 256, 7160),     # seven-wave x 32-row expert workgroups, ragged last tile
                                       (256, 8, 2, 384, 4090)])    # eight-wave x 16-row expert workgroups, ragged last tile
def test_moe_gemm_and_combine(B, T, E, k, H, N):
    g = gen(T + E + N)
    A = WL.randn_bf16(g, T, H)
    W = WL.randn_bf16(g, E, N, H, std=0.05)
    lg = torch.randn(T, E, generator=g, dtype=torch.float32)
    if E == 8 and T == 9:
        lg[:, 5] = -100.0                                  # an expert nobody selects
    idx, w, counts, offsets, perm = O.moe_route(lg.numpy(), k)
    rows = T * k
    Cd = torch.full((rows, N), 3.0, dtype=torch.bfloat16, device=DEV)
    permd, offd = dev(torch.tensor(perm)), dev(torch.tensor(offsets))
    B.ts_moe_gemm(dev(A), permd, k, dev(W), offd, Cd, rows, E, N, H)
    ref = O.moe_gemm(WL.as_f64(A), perm // k, WL.as_f64(W), offsets)
    assert_close(Cd, ref, f"moe gemm T={T} E={E}")
    # identity row map (already grouped input)
    Ag = WL.randn_bf16(g, rows, H)
    B.ts_moe_gemm(dev(Ag), None, 1, dev(W), offd, Cd, rows, E, N, H)
    ref2 = O.moe_gemm(WL.as_f64(Ag), None, WL.as_f64(W), offsets)
    assert_close(Cd, ref2, "moe gemm identity map")
    if N % 8 == 0:
        res = WL.randn_bf16(g, T, N)
        out = torch.empty(T, N, dtype=torch.bfloat16, device=DEV)
        inv = torch.empty(rows, dtype=torch.int32, device=DEV)
        wd = dev(torch.tensor(w, dtype=torch.float32))
        B.ts_moe_combine(Cd, permd, wd, dev(res), out, inv, T, k, N)
        refc = O.moe_combine(to_np(Cd), perm, w.astype(np.float32), WL.as_f64(res), T, k)
        assert_close(out, refc, "moe combine")
