"""CPU oracle for the decoder-layer hot path (TEST INFRASTRUCTURE, not product).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this.  It shares no code with the HIP path and never imports it.

What it is: the plain mathematical definition of each kernel of one LLM
decoder layer, written out in numpy float64, one function per kernel plus the
whole-layer composition.  The paper (Sec. 2.3, Sec. 3.1) treats these kernels
as opaque framework kernels and characterises them only by regime (skinny
matrix products bandwidth-bound, tiled prefill attention compute-bound); it
prints no formula for them.  The definitions used here are therefore the
standard Llama/Mixtral-style ones that the benchmark configurations name
(RMSNorm, y = A W^T projections, rotate-half RoPE, GQA softmax attention over
a contiguous KV cache, SwiGLU, top-k softmax routing); each function below
states the reading it takes.  `np.matmul` serves as a library step for the
dense contractions; there is no blocking, fusion or reordering here.

Arithmetic: float64 everywhere.  Inputs are bf16-representable values widened
exactly; intermediates are never rounded unless `round_boundaries=True`, which
rounds every kernel-boundary buffer (the buffers the method would ship between
GPUs, Sec. 3.1 data-dependency graph) to bf16 the way the GPU path stores them.

Pins (tests/test_oracle_pins.py): brute-force scalar loops on tiny cases,
closed forms (2-D rotation, unit RMS, single-key attention, uniform attention),
invariances (softmax shift, RoPE relative position, causality), cross-checks
between the decode and prefill attention paths, MoE == dense when all experts
are equal, hand-built routing ties.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------
# bf16 rounding used ONLY by the round_boundaries mode (own implementation).
# ----------------------------------------------------------------------------
def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bf16 (ties to even), return float64."""
    f = np.asarray(a, dtype=np.float32)          # fp64 -> fp32 (RNE)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(F64).reshape(np.shape(a))


# ----------------------------------------------------------------------------
# Kernels
# ----------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, gamma: np.ndarray, eps: float) -> np.ndarray:
    """y[t,i] = x[t,i] / sqrt(mean_j x[t,j]^2 + eps) * gamma[i]."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gamma, F64)


def gemm(A: np.ndarray, W: np.ndarray, residual: np.ndarray | None = None) -> np.ndarray:
    """C[m,n] = sum_c A[m,c] * W[n,c]  (+ residual[m,n]).  W is stored [N,K]."""
    C = np.matmul(np.asarray(A, F64), np.asarray(W, F64).T)
    if residual is not None:
        C = C + np.asarray(residual, F64)
    return C


def rope(u: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate-half rotary embedding on u[T, heads, d].

    For i in [0, d/2): theta_i = base^(-2i/d), phi = pos * theta_i,
      u'[i]       = u[i] cos(phi) - u[i + d/2] sin(phi)
      u'[i + d/2] = u[i + d/2] cos(phi) + u[i] sin(phi)
    """
    u = np.asarray(u, F64)
    T, nh, d = u.shape
    half = d // 2
    i = np.arange(half, dtype=F64)
    theta = base ** (-2.0 * i / d)
    phi = np.asarray(pos, F64)[:, None] * theta[None, :]       # [T, half]
    c = np.cos(phi)[:, None, :]
    s = np.sin(phi)[:, None, :]
    lo, hi = u[..., :half], u[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def kv_append(kcache: np.ndarray, vcache: np.ndarray, k: np.ndarray, v: np.ndarray,
              seq_id: np.ndarray, pos: np.ndarray) -> None:
    """In place: K[b, h, p, :] = k[t, h, :], V[b, h, p, :] = v[t, h, :] with b=seq_id[t], p=pos[t]."""
    for t in range(k.shape[0]):
        b, p = int(seq_id[t]), int(pos[t])
        kcache[b, :, p, :] = k[t]
        vcache[b, :, p, :] = v[t]


def _softmax_av(s: np.ndarray, V: np.ndarray) -> np.ndarray:
    m = np.max(s)
    e = np.exp(s - m)
    p = e / np.sum(e)
    return p @ V


def attention_decode(q: np.ndarray, kcache: np.ndarray, vcache: np.ndarray,
                     seq_lens: np.ndarray, scale: float) -> np.ndarray:
    """One query token per sequence.  q[B, nq, d]; caches [B, nkv, Lcap, d].

    Query head h reads kv head h // (nq/nkv) and attends keys j in [0, seq_lens[b]).
    s_j = scale * <q, K_j>,  p = softmax(s),  o = sum_j p_j V_j.
    """
    q = np.asarray(q, F64)
    B, nq, d = q.shape
    nkv = kcache.shape[1]
    g = nq // nkv
    out = np.zeros((B, nq, d), F64)
    for b in range(B):
        L = int(seq_lens[b])
        if L <= 0:
            continue                      # no key: output defined as zero
        for kvh in range(nkv):
            K = np.asarray(kcache[b, kvh, :L, :], F64)     # widened once per kv head
            V = np.asarray(vcache[b, kvh, :L, :], F64)
            for h in range(kvh * g, (kvh + 1) * g):        # the g query heads that share it
                s = scale * (K @ q[b, h])
                out[b, h] = _softmax_av(s, V)
    return out


def attention_prefill(q: np.ndarray, k: np.ndarray, v: np.ndarray, cu_seqlens: np.ndarray,
                      scale: float, causal: bool = True) -> np.ndarray:
    """Packed sequences.  q[T, nq, d], k/v[T, nkv, d]; sequence s owns rows cu[s]:cu[s+1].

    Token at in-sequence index i attends j <= i of its own sequence (all j if not causal).
    """
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    v = np.asarray(v, F64)
    T, nq, d = q.shape
    nkv = k.shape[1]
    g = nq // nkv
    out = np.zeros((T, nq, d), F64)
    for s_ in range(len(cu_seqlens) - 1):
        a, e = int(cu_seqlens[s_]), int(cu_seqlens[s_ + 1])
        n = e - a
        if n <= 0:
            continue
        for h in range(nq):
            S = scale * (q[a:e, h, :] @ k[a:e, h // g, :].T)       # [n, n]
            if causal:
                S = np.where(np.tril(np.ones((n, n), bool)), S, -np.inf)
            S = S - np.max(S, axis=1, keepdims=True)
            P = np.exp(S)
            P = P / np.sum(P, axis=1, keepdims=True)
            out[a:e, h, :] = P @ v[a:e, h // g, :]
    return out


def swiglu(gate_up: np.ndarray) -> np.ndarray:
    """gate_up[T, 2F] = [gate | up]  ->  silu(gate) * up,  silu(z) = z / (1 + exp(-z))."""
    gu = np.asarray(gate_up, F64)
    F = gu.shape[-1] // 2
    gate, up = gu[..., :F], gu[..., F:]
    return gate / (1.0 + np.exp(-gate)) * up


def moe_route(logits: np.ndarray, k: int):
    """Top-k routing from fp32 logits[T, E].

    Selection compares the logits exactly as given (float32 values, no
    arithmetic), larger first, ties to the lower expert index; slot order is
    the selection order.  Weights are the softmax over the k selected logits.
    counts[e] = assignments to e; offsets = exclusive prefix sum; perm lists the
    flat assignment ids t*k+s grouped by expert, ascending inside an expert.
    """
    lg = np.asarray(logits, np.float32)
    T, E = lg.shape
    idx = np.zeros((T, k), np.int32)
    w = np.zeros((T, k), F64)
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-float(lg[t, e]), e))[:k]
        idx[t] = order
        sel = lg[t, order].astype(F64)
        ex = np.exp(sel - sel[0])
        w[t] = ex / np.sum(ex)
    counts = np.zeros(E, np.int32)
    for e in idx.reshape(-1):
        counts[e] += 1
    offsets = np.zeros(E + 1, np.int32)
    offsets[1:] = np.cumsum(counts)
    flat = idx.reshape(-1)
    perm = np.array([a for e in range(E) for a in range(T * k) if flat[a] == e], np.int32)
    return idx, w, counts, offsets, perm


def moe_gemm(A: np.ndarray, row_map, W: np.ndarray, offsets: np.ndarray) -> np.ndarray:
    """Grouped product.  Output row r in [offsets[e], offsets[e+1]) is A[row_map[r]] @ W[e]^T.

    row_map None means identity (A already in grouped order).
    """
    A = np.asarray(A, F64)
    E, N, K = W.shape
    rows = int(offsets[E])
    C = np.zeros((rows, N), F64)
    for e in range(E):
        a, b = int(offsets[e]), int(offsets[e + 1])
        if b > a:
            src = A[a:b] if row_map is None else A[np.asarray(row_map[a:b], np.int64)]
            C[a:b] = src @ np.asarray(W[e], F64).T
    return C


def moe_combine(y: np.ndarray, perm: np.ndarray, topk_w: np.ndarray,
                residual: np.ndarray | None, T: int, k: int) -> np.ndarray:
    """out[t] = residual[t] + sum_s w[t,s] * y[r(t,s)], where perm[r(t,s)] = t*k+s."""
    y = np.asarray(y, F64)
    H = y.shape[1]
    out = np.zeros((T, H), F64) if residual is None else np.array(residual, F64)
    wflat = np.asarray(topk_w, F64).reshape(-1)
    for r in range(T * k):
        a = int(perm[r])
        out[a // k] += wflat[a] * y[r]
    return out


# ----------------------------------------------------------------------------
# Whole layer
# ----------------------------------------------------------------------------
BOUNDARY_ORDER_DENSE = ("h1", "qkv", "attn", "x2", "h2", "gate_up", "act", "out")
BOUNDARY_ORDER_MOE = ("h1", "qkv", "attn", "x2", "h2", "logits", "gate_up", "act", "y", "out")


def layer_forward(shape, weights: dict, io: dict, mode: str, round_boundaries: bool = False,
                  forced_route=None, perturb=None) -> dict:
    """Full decoder layer; returns every kernel-boundary tensor plus 'out'.

    perturb: optional {boundary name: callable(array) -> array}, applied to that kernel's result before it is
    stored (and, with round_boundaries, before it is rounded).  The default (None) changes nothing.  Tests use
    it to measure how a kernel-sized disturbance of one buffer travels through the bf16 roundings of the
    buffers after it, which is what an end-to-end comparison of two bf16 pipelines sees.

    shape: object with H, nq, nkv, d, F, E, k, eps, rope_base.
    weights: gamma1, w_qkv, w_o, gamma2, w_gate_up, w_down (+ w_router for MoE), float arrays.
    io: x[T,H], pos[T], seq_id[T], kcache, vcache (float arrays, modified in place by the
        append), and seq_lens[B] (decode: keys attended after the append) or cu_seqlens (prefill).
    forced_route: optional (idx, w) to teacher-force the routing decision.
    """
    s = shape
    rnd = round_bf16 if round_boundaries else (lambda a: a)
    perturb = perturb or {}
    x = np.asarray(io["x"], F64)
    T = x.shape[0]
    scale = 1.0 / np.sqrt(s.d)
    r = {}
    def R(a, name=None):
        if name in perturb:
            a = perturb[name](a)
        return rnd(a)

    r["h1"] = R(rmsnorm(x, weights["gamma1"], s.eps), "h1")
    qkv = gemm(r["h1"], weights["w_qkv"])
    if round_boundaries:
        qkv = R(qkv)                      # the projection's own output buffer
    nqd, nkd = s.nq * s.d, s.nkv * s.d
    q = qkv[:, :nqd].reshape(T, s.nq, s.d)
    kk = qkv[:, nqd:nqd + nkd].reshape(T, s.nkv, s.d)
    vv = qkv[:, nqd + nkd:].reshape(T, s.nkv, s.d)
    q = R(rope(q, io["pos"], s.rope_base))
    kk = R(rope(kk, io["pos"], s.rope_base))
    r["qkv"] = np.concatenate([q.reshape(T, -1), kk.reshape(T, -1), vv.reshape(T, -1)], axis=1)
    kv_append(io["kcache"], io["vcache"], kk, vv, io["seq_id"], io["pos"])
    if mode == "decode":
        attn = attention_decode(q, io["kcache"], io["vcache"], io["seq_lens"], scale)
    else:
        attn = attention_prefill(q, kk, vv, io["cu_seqlens"], scale, causal=True)
    r["attn"] = R(attn.reshape(T, nqd), "attn")
    r["x2"] = R(gemm(r["attn"], weights["w_o"], residual=x), "x2")
    r["h2"] = R(rmsnorm(r["x2"], weights["gamma2"], s.eps), "h2")
    if s.E == 0:
        r["gate_up"] = R(gemm(r["h2"], weights["w_gate_up"]), "gate_up")
        r["act"] = R(swiglu(r["gate_up"]), "act")
        r["out"] = R(gemm(r["act"], weights["w_down"], residual=r["x2"]), "out")
    else:
        logits = gemm(r["h2"], weights["w_router"])
        r["logits"] = logits.astype(np.float32).astype(F64) if round_boundaries else logits
        idx, w, counts, offsets, perm = moe_route(r["logits"].astype(np.float32), s.k)
        if forced_route is not None:
            idx = np.asarray(forced_route[0], np.int32)
            w = np.asarray(forced_route[1], F64)
            _, _, counts, offsets, perm = _regroup(idx, s.E)
        r["topk_idx"], r["topk_w"], r["counts"], r["offsets"], r["perm"] = idx, w, counts, offsets, perm
        row_map = perm // s.k
        r["gate_up"] = R(moe_gemm(r["h2"], row_map, weights["w_gate_up"], offsets), "gate_up")
        r["act"] = R(swiglu(r["gate_up"]), "act")
        r["y"] = R(moe_gemm(r["act"], None, weights["w_down"], offsets), "y")
        r["out"] = R(moe_combine(r["y"], perm, w, r["x2"], T, s.k), "out")
    return r


def _regroup(idx: np.ndarray, E: int):
    T, k = idx.shape
    counts = np.zeros(E, np.int32)
    for e in idx.reshape(-1):
        counts[e] += 1
    offsets = np.zeros(E + 1, np.int32)
    offsets[1:] = np.cumsum(counts)
    flat = idx.reshape(-1)
    perm = np.array([a for e in range(E) for a in range(T * k) if flat[a] == e], np.int32)
    return idx, None, counts, offsets, perm


def boundary_stream(result: dict, moe: bool, mask: int = ~0) -> np.ndarray:
    """Concatenate the flagged boundary tensors, in kernel order, as one flat float64 array.

    Mirrors what the pipelined step ships per micro-batch: bit i of `mask`
    selects the i-th boundary of BOUNDARY_ORDER_*.
    """
    order = BOUNDARY_ORDER_MOE if moe else BOUNDARY_ORDER_DENSE
    parts = [np.asarray(result[n], F64).reshape(-1) for i, n in enumerate(order) if (mask >> i) & 1]
    return np.concatenate(parts) if parts else np.zeros(0, F64)
