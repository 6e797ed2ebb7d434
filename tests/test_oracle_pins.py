"""Pins for the CPU oracle: brute force, closed forms, invariants.

None of these call the HIP path.  Each check is chosen so that a plausible slip
in oracle/decoder_layer.py (dropped term, wrong sign or index, transposed
operand, wrong head mapping) fails at least one of them.  The brute-force
references below are scalar Python loops written from the definitions, not
from the oracle's vectorised code.
"""
import math

import numpy as np
import pytest

from oracle import decoder_layer as O

rng = np.random.default_rng(1234)


# ------------------------------------------------------------------ bf16 rounding
def test_round_bf16_known_values():
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1.0 and 1+2^-7: ties to even -> 1.0
    assert O.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    # 1 + 3*2^-8 is halfway between 1+2^-7 and 1+2^-6: ties to even -> 1+2^-6
    assert O.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert O.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    v = np.array([0.0, -2.5, 3.0e38, 1e-3])
    r = O.round_bf16(v)
    assert r[0] == 0.0 and r[1] == -2.5
    assert abs(r[3] - 1e-3) <= 1e-3 * 2.0 ** -8
    # idempotent
    assert np.array_equal(O.round_bf16(r), r)


def test_round_bf16_matches_torch():
    torch = pytest.importorskip("torch")
    v = rng.standard_normal(4096) * np.exp(rng.uniform(-20, 20, 4096))
    want = torch.tensor(v, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_bf16(v), want)


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_unit_rms_and_scale_invariance():
    x = rng.standard_normal((5, 64))
    y = O.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=1)), 1.0, atol=1e-14)
    y2 = O.rmsnorm(7.5 * x, np.ones(64), 0.0)
    assert np.allclose(y, y2, atol=1e-14)


def test_rmsnorm_constant_row_and_bruteforce():
    g = rng.standard_normal(8)
    y = O.rmsnorm(np.full((1, 8), -3.0), g, 0.0)
    assert np.allclose(y[0], -g, atol=1e-15)
    x = rng.standard_normal((3, 8))
    eps = 1e-2
    y = O.rmsnorm(x, g, eps)
    for t in range(3):
        ms = sum(x[t, j] ** 2 for j in range(8)) / 8
        for i in range(8):
            assert abs(y[t, i] - x[t, i] / math.sqrt(ms + eps) * g[i]) < 1e-14


# ------------------------------------------------------------------ GEMM
def test_gemm_bruteforce_nonsquare():
    M, N, K = 3, 5, 7
    A = rng.standard_normal((M, K))
    W = rng.standard_normal((N, K))
    R = rng.standard_normal((M, N))
    C = O.gemm(A, W, R)
    assert C.shape == (M, N)
    for m in range(M):
        for n in range(N):
            acc = R[m, n]
            for c in range(K):
                acc += A[m, c] * W[n, c]
            assert abs(C[m, n] - acc) < 1e-13


def test_gemm_identity_linearity_tail():
    A = rng.standard_normal((4, 16))
    assert np.array_equal(O.gemm(A, np.eye(16)), A)
    W = rng.standard_normal((6, 688))           # the odd inner width of the tiny layer
    A1, A2 = rng.standard_normal((2, 688)), rng.standard_normal((2, 688))
    assert np.allclose(O.gemm(A1 + 2 * A2, W), O.gemm(A1, W) + 2 * O.gemm(A2, W), atol=1e-11)
    # a selector row picks one column of W^T
    e = np.zeros((1, 688)); e[0, 687] = 1.0
    assert np.array_equal(O.gemm(e, W)[0], W[:, 687])


# ------------------------------------------------------------------ RoPE
def test_rope_position_zero_is_identity_and_norms():
    u = rng.standard_normal((3, 2, 8))
    assert np.allclose(O.rope(u, np.zeros(3), 10000.0), u, atol=0)
    r = O.rope(u, np.array([1, 17, 4000]), 10000.0)
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(u, axis=-1), atol=1e-13)
    # each (i, i+d/2) pair keeps its own norm
    assert np.allclose(r[..., :4] ** 2 + r[..., 4:] ** 2, u[..., :4] ** 2 + u[..., 4:] ** 2, atol=1e-12)


def test_rope_2d_closed_form_and_direction():
    # d = 2: a single pair, theta_0 = 1, so position p rotates the plane by p radians (counter-clockwise)
    u = np.array([[[1.0, 0.0]]])
    r = O.rope(u, np.array([1]), 12345.0)
    assert np.allclose(r[0, 0], [math.cos(1.0), math.sin(1.0)], atol=1e-15)
    u = np.array([[[0.0, 1.0]]])
    r = O.rope(u, np.array([2]), 7.0)
    assert np.allclose(r[0, 0], [-math.sin(2.0), math.cos(2.0)], atol=1e-15)


def test_rope_frequencies_bruteforce():
    d, base = 8, 100.0
    u = rng.standard_normal((2, 3, d))
    pos = np.array([5, 9])
    r = O.rope(u, pos, base)
    for t in range(2):
        for h in range(3):
            for i in range(d // 2):
                th = base ** (-2.0 * i / d)
                c, s = math.cos(pos[t] * th), math.sin(pos[t] * th)
                a, b = u[t, h, i], u[t, h, i + d // 2]
                assert abs(r[t, h, i] - (a * c - b * s)) < 1e-14
                assert abs(r[t, h, i + d // 2] - (b * c + a * s)) < 1e-14


def test_rope_relative_position_property():
    d = 16
    q = rng.standard_normal((1, 1, d)); k = rng.standard_normal((1, 1, d))
    def dot(m, n):
        return float(np.sum(O.rope(q, np.array([m]), 10000.0) * O.rope(k, np.array([n]), 10000.0)))
    assert abs(dot(10, 3) - dot(107, 100)) < 1e-11
    assert abs(dot(10, 3) - dot(3, 10)) > 1e-3       # and it does depend on the sign of m-n


# ------------------------------------------------------------------ attention
def _attn_bruteforce(q, K, V, scale):
    L, d = K.shape
    s = [scale * sum(q[c] * K[j, c] for c in range(d)) for j in range(L)]
    m = max(s)
    e = [math.exp(v - m) for v in s]
    z = sum(e)
    return [sum(e[j] / z * V[j, c] for j in range(L)) for c in range(V.shape[1])]


def test_attention_decode_bruteforce_gqa_and_lengths():
    B, nq, nkv, d, Lcap = 2, 4, 2, 4, 6
    q = rng.standard_normal((B, nq, d))
    kc = rng.standard_normal((B, nkv, Lcap, d))
    vc = rng.standard_normal((B, nkv, Lcap, d))
    lens = np.array([6, 3])
    kc[1, :, 3:] = np.nan; vc[1, :, 3:] = np.nan       # must not be read
    out = O.attention_decode(q, kc, vc, lens, 0.37)
    for b in range(B):
        for h in range(nq):
            ref = _attn_bruteforce(q[b, h], kc[b, h // 2, :lens[b]], vc[b, h // 2, :lens[b]], 0.37)
            assert np.allclose(out[b, h], ref, atol=1e-13)


def test_attention_single_key_identical_keys_shift():
    d = 8
    q = rng.standard_normal((1, 2, d))
    kc = rng.standard_normal((1, 1, 5, d)); vc = rng.standard_normal((1, 1, 5, d))
    o = O.attention_decode(q, kc, vc, np.array([1]), 1.0)
    assert np.allclose(o[0, 0], vc[0, 0, 0]) and np.allclose(o[0, 1], vc[0, 0, 0])
    kc2 = np.broadcast_to(kc[:, :, :1], kc.shape).copy()        # all keys identical -> uniform weights
    o = O.attention_decode(q, kc2, vc, np.array([5]), 1.0)
    assert np.allclose(o[0, 0], vc[0, 0].mean(axis=0), atol=1e-13)
    # adding a constant to every score (k += c*q/|q|^2 adds c to each <q,k>) changes nothing
    qh = q[0, 0]
    o1 = O.attention_decode(q[:, :1], kc, vc, np.array([5]), 1.0)
    o2 = O.attention_decode(q[:, :1], kc + 3.0 * qh / np.dot(qh, qh), vc, np.array([5]), 1.0)
    assert np.allclose(o1, o2, atol=1e-12)
    assert O.attention_decode(q, kc, vc, np.array([0]), 1.0).sum() == 0.0


def test_softmax_rows_sum_to_one_via_constant_v():
    # with V == 1 everywhere the output is sum_j p_j, which must be exactly 1 up to rounding
    q = rng.standard_normal((3, 4, 8)) * 5
    kc = rng.standard_normal((3, 2, 9, 8)); vc = np.ones((3, 2, 9, 8))
    o = O.attention_decode(q, kc, vc, np.array([9, 4, 1]), 0.5)
    assert np.allclose(o, 1.0, atol=1e-14)
    k = rng.standard_normal((7, 2, 8))
    o = O.attention_prefill(rng.standard_normal((7, 4, 8)), k, np.ones((7, 2, 8)), np.array([0, 3, 7]), 0.5)
    assert np.allclose(o, 1.0, atol=1e-14)


def test_attention_prefill_bruteforce_causal_two_sequences():
    T, nq, nkv, d = 7, 4, 2, 4
    q = rng.standard_normal((T, nq, d)); k = rng.standard_normal((T, nkv, d)); v = rng.standard_normal((T, nkv, d))
    cu = np.array([0, 3, 7])
    out = O.attention_prefill(q, k, v, cu, 0.5, causal=True)
    for s in range(2):
        a, e = cu[s], cu[s + 1]
        for i in range(a, e):
            for h in range(nq):
                ref = _attn_bruteforce(q[i, h], k[a:i + 1, h // 2], v[a:i + 1, h // 2], 0.5)
                assert np.allclose(out[i, h], ref, atol=1e-13)
    full = O.attention_prefill(q, k, v, cu, 0.5, causal=False)
    ref = _attn_bruteforce(q[4, 1], k[3:7, 0], v[3:7, 0], 0.5)
    assert np.allclose(full[4, 1], ref, atol=1e-13)


def test_attention_causality_and_sequence_isolation():
    T, nq, nkv, d = 8, 2, 1, 4
    q = rng.standard_normal((T, nq, d)); k = rng.standard_normal((T, nkv, d)); v = rng.standard_normal((T, nkv, d))
    cu = np.array([0, 5, 8])
    base = O.attention_prefill(q, k, v, cu, 1.0)
    k2, v2 = k.copy(), v.copy()
    k2[3:5] += 10.0; v2[3:5] -= 7.0                   # future of token 2, inside sequence 0
    pert = O.attention_prefill(q, k2, v2, cu, 1.0)
    assert np.array_equal(base[:3], pert[:3])         # tokens 0..2 untouched
    assert not np.allclose(base[3:5], pert[3:5])
    assert np.array_equal(base[5:], pert[5:])         # other sequence untouched


def test_decode_equals_last_row_of_prefill():
    L, nq, nkv, d = 6, 4, 2, 8
    q = rng.standard_normal((L + 1, nq, d)); k = rng.standard_normal((L + 1, nkv, d)); v = rng.standard_normal((L + 1, nkv, d))
    pre = O.attention_prefill(q, k, v, np.array([0, L + 1]), 0.3)
    kc = np.transpose(k, (1, 0, 2))[None].copy(); vc = np.transpose(v, (1, 0, 2))[None].copy()
    dec = O.attention_decode(q[L:L + 1], kc, vc, np.array([L + 1]), 0.3)
    assert np.allclose(dec[0], pre[L], atol=1e-13)


# ------------------------------------------------------------------ SwiGLU
def test_swiglu_pointwise():
    F = 5
    g = np.array([[0.0, 30.0, -30.0, 1.0, -1.0]]); u = np.array([[3.0, 2.0, 2.0, 0.0, 4.0]])
    y = O.swiglu(np.concatenate([g, u], axis=1))[0]
    assert y[0] == 0.0                                   # silu(0) = 0
    assert abs(y[1] - 60.0) < 1e-9                       # gate -> +large: gate*up
    assert abs(y[2]) < 1e-9                              # gate -> -large: 0
    assert y[3] == 0.0                                   # up = 0
    assert abs(y[4] - (-1.0 / (1.0 + math.e)) * 4.0) < 1e-15
    gu = rng.standard_normal((3, 2 * F))
    y = O.swiglu(gu)
    for t in range(3):
        for f in range(F):
            z = gu[t, f]
            assert abs(y[t, f] - z / (1 + math.exp(-z)) * gu[t, F + f]) < 1e-15


# ------------------------------------------------------------------ MoE
def test_moe_route_ties_and_bookkeeping():
    lg = np.array([[1.0, 3.0, 3.0, 0.0],      # tie between experts 1,2 -> 1 first
                   [5.0, 5.0, 5.0, 5.0],      # all tied -> 0,1
                   [0.0, -1.0, 2.0, 1.0],     # -> 2,3
                   [-2.0, -1.0, -3.0, -1.0]], np.float32)   # tie 1,3 -> 1,3
    idx, w, counts, offsets, perm = O.moe_route(lg, 2)
    assert idx.tolist() == [[1, 2], [0, 1], [2, 3], [1, 3]]
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-15)
    assert np.allclose(w[0], [0.5, 0.5]) and np.allclose(w[2], [math.e / (1 + math.e), 1 / (1 + math.e)])
    assert counts.tolist() == [1, 3, 2, 2] and offsets.tolist() == [0, 1, 4, 6, 8]
    assert perm.tolist() == [2, 0, 3, 6, 1, 4, 5, 7]
    assert sorted(perm.tolist()) == list(range(8))
    idx1, w1, c1, _, _ = O.moe_route(lg, 1)
    assert np.array_equal(w1, np.ones((4, 1))) and c1.sum() == 4


def test_moe_route_random_properties():
    T, E, k = 64, 8, 2
    lg = rng.standard_normal((T, E)).astype(np.float32)
    idx, w, counts, offsets, perm = O.moe_route(lg, k)
    assert counts.sum() == T * k and offsets[-1] == T * k
    assert sorted(perm.tolist()) == list(range(T * k))
    for t in range(T):
        srt = np.sort(lg[t])[::-1]
        assert lg[t, idx[t, 0]] == srt[0] and lg[t, idx[t, 1]] == srt[1]
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert all(idx.reshape(-1)[a] == e for a in seg) and list(seg) == sorted(seg)


def test_moe_gemm_and_combine_bruteforce():
    T, k, E, H, N = 5, 2, 3, 4, 6
    A = rng.standard_normal((T, H)); W = rng.standard_normal((E, N, H))
    lg = rng.standard_normal((T, E)).astype(np.float32)
    idx, w, counts, offsets, perm = O.moe_route(lg, k)
    C = O.moe_gemm(A, perm // k, W, offsets)
    for r in range(T * k):
        t = perm[r] // k; e = idx.reshape(-1)[perm[r]]
        for n in range(N):
            assert abs(C[r, n] - sum(A[t, c] * W[e, n, c] for c in range(H))) < 1e-13
    res = rng.standard_normal((T, N))
    out = O.moe_combine(C, perm, w, res, T, k)
    for t in range(T):
        for n in range(N):
            acc = res[t, n]
            for s in range(k):
                e = idx[t, s]
                acc += w[t, s] * sum(A[t, c] * W[e, n, c] for c in range(H))
            assert abs(out[t, n] - acc) < 1e-13


# ------------------------------------------------------------------ whole layer
class _S:
    def __init__(self, **kw):
        self.__dict__.update(kw)


def _tiny_layer(E=0, k=0, T=3, L=4):
    s = _S(H=16, nq=4, nkv=2, d=4, F=12, E=E, k=k, eps=1e-5, rope_base=10000.0)
    w = {"gamma1": 1 + 0.1 * rng.standard_normal(s.H), "gamma2": 1 + 0.1 * rng.standard_normal(s.H),
         "w_qkv": 0.3 * rng.standard_normal(((s.nq + 2 * s.nkv) * s.d, s.H)),
         "w_o": 0.3 * rng.standard_normal((s.H, s.nq * s.d))}
    if E:
        w["w_router"] = rng.standard_normal((E, s.H))
        w["w_gate_up"] = 0.3 * rng.standard_normal((E, 2 * s.F, s.H))
        w["w_down"] = 0.3 * rng.standard_normal((E, s.H, s.F))
    else:
        w["w_gate_up"] = 0.3 * rng.standard_normal((2 * s.F, s.H))
        w["w_down"] = 0.3 * rng.standard_normal((s.H, s.F))
    io = {"x": rng.standard_normal((T, s.H)), "pos": np.full(T, L), "seq_id": np.arange(T),
          "seq_lens": np.full(T, L + 1),
          "kcache": rng.standard_normal((T, s.nkv, L + 1, s.d)), "vcache": rng.standard_normal((T, s.nkv, L + 1, s.d))}
    return s, w, io


def _copy_io(io):
    return {k: np.array(v) for k, v in io.items()}


def test_layer_zero_projections_is_identity():
    s, w, io = _tiny_layer()
    w["w_o"][:] = 0; w["w_down"][:] = 0
    r = O.layer_forward(s, w, io, "decode")
    assert np.array_equal(r["out"], io["x"])


def test_layer_dense_bruteforce_one_token():
    """Scalar-loop evaluation of the whole dense decode layer for one token."""
    s, w, io = _tiny_layer(T=1, L=3)
    io0 = _copy_io(io)
    r = O.layer_forward(s, w, io, "decode")
    x = io0["x"][0]; H, d = s.H, s.d
    ms = sum(v * v for v in x) / H
    h1 = [x[i] / math.sqrt(ms + s.eps) * w["gamma1"][i] for i in range(H)]
    qkv = [sum(h1[c] * w["w_qkv"][n, c] for c in range(H)) for n in range((s.nq + 2 * s.nkv) * d)]
    def rot(vec, p):
        o = list(vec)
        for i in range(d // 2):
            th = s.rope_base ** (-2.0 * i / d)
            c_, s_ = math.cos(p * th), math.sin(p * th)
            o[i] = vec[i] * c_ - vec[i + d // 2] * s_
            o[i + d // 2] = vec[i + d // 2] * c_ + vec[i] * s_
        return o
    p = 3
    qh = [rot(qkv[h * d:(h + 1) * d], p) for h in range(s.nq)]
    kh = [rot(qkv[s.nq * d + h * d: s.nq * d + (h + 1) * d], p) for h in range(s.nkv)]
    vh = [qkv[(s.nq + s.nkv) * d + h * d:(s.nq + s.nkv) * d + (h + 1) * d] for h in range(s.nkv)]
    attn = []
    for h in range(s.nq):
        kvh = h // (s.nq // s.nkv)
        K = np.vstack([io0["kcache"][0, kvh, :3], np.array(kh[kvh])])
        V = np.vstack([io0["vcache"][0, kvh, :3], np.array(vh[kvh])])
        attn += _attn_bruteforce(qh[h], K, V, 1 / math.sqrt(d))
    x2 = [x[i] + sum(attn[c] * w["w_o"][i, c] for c in range(s.nq * d)) for i in range(H)]
    ms2 = sum(v * v for v in x2) / H
    h2 = [x2[i] / math.sqrt(ms2 + s.eps) * w["gamma2"][i] for i in range(H)]
    gu = [sum(h2[c] * w["w_gate_up"][n, c] for c in range(H)) for n in range(2 * s.F)]
    act = [gu[f] / (1 + math.exp(-gu[f])) * gu[s.F + f] for f in range(s.F)]
    out = [x2[i] + sum(act[f] * w["w_down"][i, f] for f in range(s.F)) for i in range(H)]
    assert np.allclose(r["out"][0], out, atol=1e-12)
    assert np.allclose(r["x2"][0], x2, atol=1e-12)
    assert np.allclose(io["kcache"][0, :, 3, :], np.array(kh), atol=1e-13)   # appended rotated K
    assert np.allclose(io["vcache"][0, :, 3, :], np.array(vh), atol=1e-13)


def test_layer_moe_with_identical_experts_equals_dense():
    s, w, io = _tiny_layer()
    sm, wm, _ = _tiny_layer(E=4, k=2)
    for n in ("gamma1", "gamma2", "w_qkv", "w_o"):
        wm[n] = w[n]
    wm["w_gate_up"] = np.broadcast_to(w["w_gate_up"], (4,) + w["w_gate_up"].shape).copy()
    wm["w_down"] = np.broadcast_to(w["w_down"], (4,) + w["w_down"].shape).copy()
    rd = O.layer_forward(s, w, _copy_io(io), "decode")
    rm = O.layer_forward(sm, wm, _copy_io(io), "decode")
    assert np.allclose(rd["out"], rm["out"], atol=1e-12)
    assert np.allclose(rm["topk_w"].sum(axis=1), 1.0)


def test_layer_prefill_then_decode_consistency():
    """Prefill L+1 tokens; its last token must equal decoding that token over the cache prefill wrote."""
    s, w, _ = _tiny_layer()
    L = 5
    x = rng.standard_normal((L + 1, s.H))
    def fresh():
        return np.zeros((1, s.nkv, L + 1, s.d)), np.zeros((1, s.nkv, L + 1, s.d))
    kc, vc = fresh()
    io_p = {"x": x, "pos": np.arange(L + 1), "seq_id": np.zeros(L + 1, int), "cu_seqlens": np.array([0, L + 1]),
            "kcache": kc, "vcache": vc}
    rp = O.layer_forward(s, w, io_p, "prefill")
    kc2, vc2 = fresh()
    io_p2 = {"x": x[:L], "pos": np.arange(L), "seq_id": np.zeros(L, int), "cu_seqlens": np.array([0, L]),
             "kcache": kc2, "vcache": vc2}
    O.layer_forward(s, w, io_p2, "prefill")
    io_d = {"x": x[L:], "pos": np.array([L]), "seq_id": np.array([0]), "seq_lens": np.array([L + 1]),
            "kcache": kc2, "vcache": vc2}
    rd = O.layer_forward(s, w, io_d, "decode")
    assert np.allclose(rd["out"][0], rp["out"][L], atol=1e-12)
    assert np.allclose(kc2, kc, atol=1e-13) and np.allclose(vc2, vc, atol=1e-13)


def test_round_boundaries_mode_is_close_and_bf16_valued():
    s, w, io = _tiny_layer()
    a = O.layer_forward(s, w, _copy_io(io), "decode")
    b = O.layer_forward(s, w, _copy_io(io), "decode", round_boundaries=True)
    assert np.array_equal(O.round_bf16(b["out"]), b["out"])
    rel = np.linalg.norm(a["out"] - b["out"]) / np.linalg.norm(a["out"])
    assert 0 < rel < 2e-2


def test_boundary_stream_order_and_mask():
    s, w, io = _tiny_layer()
    r = O.layer_forward(s, w, io, "decode")
    full = O.boundary_stream(r, moe=False)
    sizes = [r[n].size for n in O.BOUNDARY_ORDER_DENSE]
    assert full.size == sum(sizes)
    assert np.array_equal(full[:sizes[0]], r["h1"].reshape(-1))
    only = O.boundary_stream(r, moe=False, mask=(1 << 3) | (1 << 7))
    assert np.array_equal(only, np.concatenate([r["x2"].reshape(-1), r["out"].reshape(-1)]))
