// C ABI: argument validation, workspace planning, the whole-layer call and the pipelined
// micro-batch step.  Validation runs before the first HIP call so it can be exercised on a
// host without a GPU.
#include <cstdarg>
#include <cstdio>
#include <cmath>
#include <new>
#include <vector>
#include <algorithm>

#include "common.hpp"

namespace ts {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
int check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return TS_OK;
  snprintf(g_err, sizeof(g_err), "HIP error %d (%s) at %s", (int)e, hipGetErrorString(e), what);
  return TS_ERR_HIP;
}

// ---- per-launch profile (thread-local; events belong to the caller) ----------
struct Profile {
  hipEvent_t* events = nullptr;   // pairs: [2*i] before, [2*i+1] after launch i
  const char** names = nullptr;
  int cap = 0, used = 0;
  bool active = false;
};
static thread_local Profile g_prof;

static thread_local hipEvent_t g_stop_event = nullptr;
void arm_stop_event(hipEvent_t e) { g_stop_event = e; }
hipEvent_t take_stop_event() {
  hipEvent_t e = g_stop_event;
  g_stop_event = nullptr;
  return e;
}
bool disarm_stop_event() { return take_stop_event() != nullptr; }

void prof_begin(const char* name, hipStream_t s) {
  if (!g_prof.active || g_prof.used >= g_prof.cap) return;
  g_prof.names[g_prof.used] = name;
  (void)hipEventRecord(g_prof.events[2 * g_prof.used], s);
}
void prof_end(hipStream_t s) {
  if (!g_prof.active || g_prof.used >= g_prof.cap) return;
  (void)hipEventRecord(g_prof.events[2 * g_prof.used + 1], s);
  ++g_prof.used;
}

namespace {

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// ---- layer workspace plan ---------------------------------------------------
struct LayerPlan {
  size_t h1, qkv, attn, x2, h2, gate_up, act, y;         // boundary buffers (byte offsets)
  size_t logits, topk_idx, topk_w, counts, offsets, perm, inv;  // MoE routing buffers
  size_t scratch, scratch_bytes;
  size_t counters;                                       // int32 arrival counters (zeroed by the first kernel)
  int counter_words;
  size_t total;
  size_t bytes[TS_NB_MOE];                               // size of each boundary
};

int validate_desc(const ts_layer_desc* d, const char* who) {
  TS_REQUIRE(d != nullptr, TS_ERR_INVALID_ARG, "%s: null descriptor", who);
  TS_REQUIRE(d->H > 0 && d->nq > 0 && d->nkv > 0 && d->d > 0 && d->F > 0 && d->Lcap > 0, TS_ERR_INVALID_ARG,
             "%s: non-positive dimension", who);
  TS_REQUIRE(d->nq % d->nkv == 0, TS_ERR_INVALID_ARG, "%s: nq %% nkv != 0", who);
  TS_REQUIRE(d->mode == TS_MODE_DECODE || d->mode == TS_MODE_PREFILL, TS_ERR_INVALID_ARG, "%s: bad mode", who);
  TS_REQUIRE(d->E >= 0 && (d->E == 0 || (d->k >= 1 && d->k <= d->E)), TS_ERR_INVALID_ARG, "%s: bad E/k", who);
  TS_REQUIRE(d->H % 8 == 0 && d->H <= 32768 && d->F % 8 == 0, TS_ERR_UNSUPPORTED_SHAPE,
             "%s: H and F must be multiples of 8, H <= 32768", who);
  TS_REQUIRE(d->d == 64 || d->d == 128, TS_ERR_UNSUPPORTED_SHAPE, "%s: head dim must be 64 or 128", who);
  TS_REQUIRE(d->nq / d->nkv <= 16, TS_ERR_UNSUPPORTED_SHAPE, "%s: GQA group larger than 16", who);
  TS_REQUIRE(d->E <= 64, TS_ERR_UNSUPPORTED_SHAPE, "%s: more than 64 experts", who);
  return TS_OK;
}

LayerPlan plan_layer(const ts_layer_desc& d, int T, int B) {
  LayerPlan p{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += round_up(bytes, 256);
    return o;
  };
  const size_t nqkv = (size_t)(d.nq + 2 * d.nkv) * d.d;
  const size_t rows = d.E > 0 ? (size_t)T * d.k : (size_t)T;
  p.bytes[TS_B_H1] = (size_t)T * d.H * 2;
  p.bytes[TS_B_QKV] = (size_t)T * nqkv * 2;
  p.bytes[TS_B_ATTN] = (size_t)T * d.nq * d.d * 2;
  p.bytes[TS_B_X2] = (size_t)T * d.H * 2;
  p.bytes[TS_B_H2] = (size_t)T * d.H * 2;
  p.bytes[TS_B_GATE_UP] = rows * 2 * d.F * 2;
  p.bytes[TS_B_ACT] = rows * d.F * 2;
  if (d.E > 0) {
    p.bytes[TS_B_Y_MOE] = rows * d.H * 2;
    p.bytes[TS_B_OUT_MOE] = (size_t)T * d.H * 2;
  } else {
    p.bytes[TS_B_OUT_DENSE] = (size_t)T * d.H * 2;
  }
  p.h1 = take(p.bytes[TS_B_H1]);
  p.qkv = take(p.bytes[TS_B_QKV]);
  p.attn = take(p.bytes[TS_B_ATTN]);
  p.x2 = take(p.bytes[TS_B_X2]);
  p.h2 = take(p.bytes[TS_B_H2]);
  p.gate_up = take(p.bytes[TS_B_GATE_UP]);
  p.act = take(p.bytes[TS_B_ACT]);
  if (d.E > 0) {
    p.y = take(p.bytes[TS_B_Y_MOE]);
    p.logits = take((size_t)T * d.E * 4);
    p.topk_idx = take((size_t)T * d.k * 4);
    p.topk_w = take((size_t)T * d.k * 4);
    p.counts = take((size_t)d.E * 4);
    p.offsets = take((size_t)(d.E + 1) * 4);
    p.perm = take((size_t)T * d.k * 4);
    p.inv = take((size_t)T * d.k * 4);
  }
  size_t sc = 0;
  auto mx = [&](size_t v) { if (v > sc) sc = v; };
  mx(gemm_workspace_bytes(T, (int)nqkv, d.H));
  mx(gemm_workspace_bytes(T, d.H, d.nq * d.d));
  if (d.E > 0) {
    mx(gemm_workspace_bytes(T, d.E, d.H));
  } else {
    mx(gemm_workspace_bytes(T, 2 * d.F, d.H));
    mx(gemm_workspace_bytes(T, d.H, d.F));
  }
  if (d.mode == TS_MODE_DECODE) mx(attention_decode_workspace_bytes(B, d.nq, d.nkv, d.d, d.Lcap));
  p.scratch_bytes = sc;
  p.scratch = take(sc);
  // arrival counters of the merge inside the balanced form of decode attention (one per sequence and kv
  // head): cleared by the layer's first kernel, re-armed by the workgroup that merges
  int cw = 0;
  if (d.mode == TS_MODE_DECODE) cw = B * d.nkv;
  p.counter_words = cw;
  p.counters = take((size_t)cw * 4);
  p.total = off;
  return p;
}

size_t boundary_offset(const LayerPlan& p, const ts_layer_desc& d, int index) {
  switch (index) {
    case TS_B_H1: return p.h1;
    case TS_B_QKV: return p.qkv;
    case TS_B_ATTN: return p.attn;
    case TS_B_X2: return p.x2;
    case TS_B_H2: return p.h2;
    case TS_B_GATE_UP: return p.gate_up;
    case TS_B_ACT: return p.act;
    default: break;
  }
  if (d.E > 0 && index == TS_B_Y_MOE) return p.y;
  return (size_t)-1;  // the layer output lives in io->out
}

int validate_io(const ts_layer_desc* desc, const ts_layer_weights* w, const ts_layer_io* io, const char* who) {
  TS_REQUIRE(w != nullptr && io != nullptr, TS_ERR_INVALID_ARG, "%s: null weights/io", who);
  TS_REQUIRE(io->T >= 0 && io->B >= 0, TS_ERR_INVALID_ARG, "%s: negative T/B", who);
  TS_REQUIRE(w->gamma1 && w->w_qkv && w->w_o && w->gamma2 && w->w_gate_up && w->w_down, TS_ERR_INVALID_ARG,
             "%s: null weight pointer", who);
  TS_REQUIRE(desc->E == 0 || w->w_router != nullptr, TS_ERR_INVALID_ARG, "%s: MoE layer without router", who);
  TS_REQUIRE(io->x && io->out && io->pos && io->seq_id && io->kcache && io->vcache, TS_ERR_INVALID_ARG,
             "%s: null io pointer", who);
  TS_REQUIRE(aligned16(io->x) && aligned16(io->out) && aligned16(io->kcache) && aligned16(io->vcache), TS_ERR_INVALID_ARG,
             "%s: io pointer not 16-byte aligned", who);
  if (desc->mode == TS_MODE_DECODE) {
    TS_REQUIRE(io->seq_lens != nullptr, TS_ERR_INVALID_ARG, "%s: decode needs seq_lens", who);
    TS_REQUIRE(io->T == io->B, TS_ERR_INVALID_ARG, "%s: decode expects one token per sequence (T == B)", who);
  } else {
    TS_REQUIRE(io->cu_seqlens != nullptr && io->max_seqlen >= 0, TS_ERR_INVALID_ARG,
               "%s: prefill needs cu_seqlens and max_seqlen", who);
  }
  return TS_OK;
}

// The layer, with `pre(index)` invoked before the launch function whose last kernel completes boundary `index`
// (the place to arm a stop event) and `hook(index, ptr)` right after that boundary has been enqueued.
template <typename Pre, typename Hook>
int layer_forward_impl(const ts_layer_desc& d, const ts_layer_weights& w, const ts_layer_io& io, char* ws,
                       hipStream_t s, Pre&& pre, Hook&& hook) {
  const int T = io.T, B = io.B;
  if (T == 0) return TS_OK;
  const LayerPlan p = plan_layer(d, T, B);
  const int nqd = d.nq * d.d, nkd = d.nkv * d.d, nqkv = nqd + 2 * nkd;
  ts_bf16* h1 = reinterpret_cast<ts_bf16*>(ws + p.h1);
  ts_bf16* qkv = reinterpret_cast<ts_bf16*>(ws + p.qkv);
  ts_bf16* attn = reinterpret_cast<ts_bf16*>(ws + p.attn);
  ts_bf16* x2 = reinterpret_cast<ts_bf16*>(ws + p.x2);
  ts_bf16* h2 = reinterpret_cast<ts_bf16*>(ws + p.h2);
  ts_bf16* gate_up = reinterpret_cast<ts_bf16*>(ws + p.gate_up);
  ts_bf16* act = reinterpret_cast<ts_bf16*>(ws + p.act);
  void* scratch = ws + p.scratch;
  int32_t* counters = p.counter_words > 0 ? reinterpret_cast<int32_t*>(ws + p.counters) : nullptr;
  const float scale = 1.0f / sqrtf((float)d.d);
  int rc;
#define TS_STEP(call) do { rc = (call); if (rc != TS_OK) return rc; } while (0)
  pre(TS_B_H1);
  TS_STEP(launch_rmsnorm(io.x, w.gamma1, h1, T, d.H, d.eps, s, counters, p.counter_words));
  TS_STEP(hook(TS_B_H1, h1));
  TS_STEP(launch_gemm(h1, w.w_qkv, nullptr, qkv, false, T, nqkv, d.H, scratch, p.scratch_bytes, s));
  pre(TS_B_QKV);
  TS_STEP(launch_rope(qkv, qkv + nqd, qkv + nqd + nkd, nqkv, nqkv, io.pos, io.seq_id, w.rope_cos_sin,
                      w.rope_cos_sin ? w.rope_table_len : 0, io.kcache, io.vcache, T, d.nq, d.nkv, d.d, d.Lcap,
                      d.rope_base, s));
  TS_STEP(hook(TS_B_QKV, qkv));
  pre(TS_B_ATTN);
  if (d.mode == TS_MODE_DECODE) {
    TS_STEP(launch_attention_decode(qkv, nqkv, io.kcache, io.vcache, io.seq_lens, attn, B, d.nq, d.nkv, d.d, d.Lcap,
                                    scale, scratch, p.scratch_bytes, s, counters));
  } else {
    TS_STEP(launch_attention_prefill(qkv, qkv + nqd, qkv + nqd + nkd, nqkv, nqkv, io.cu_seqlens, attn, B, T,
                                     io.max_seqlen, d.nq, d.nkv, d.d, scale, 1, s));
  }
  TS_STEP(hook(TS_B_ATTN, attn));
  pre(TS_B_X2);
  TS_STEP(launch_gemm(attn, w.w_o, io.x, x2, false, T, d.H, nqd, scratch, p.scratch_bytes, s));
  TS_STEP(hook(TS_B_X2, x2));
  pre(TS_B_H2);
  TS_STEP(launch_rmsnorm(x2, w.gamma2, h2, T, d.H, d.eps, s));
  TS_STEP(hook(TS_B_H2, h2));
  if (d.E == 0) {
    if (gemm_mfma256_glu_supported(T, d.F, d.H)) {
      // MFMA-bound sizes: the activation is applied in the projection's epilogue (both tensors are still written)
      pre(TS_B_GATE_UP);
      TS_STEP(launch_gemm_mfma256_glu(h2, w.w_gate_up, gate_up, act, T, d.F, d.H, s));
      TS_STEP(hook(TS_B_GATE_UP, gate_up));
    } else {
      pre(TS_B_GATE_UP);
      TS_STEP(launch_gemm(h2, w.w_gate_up, nullptr, gate_up, false, T, 2 * d.F, d.H, scratch, p.scratch_bytes, s));
      TS_STEP(hook(TS_B_GATE_UP, gate_up));
      pre(TS_B_ACT);
      TS_STEP(launch_swiglu(gate_up, act, T, d.F, s));
    }
    TS_STEP(hook(TS_B_ACT, act));
    pre(TS_B_OUT_DENSE);
    TS_STEP(launch_gemm(act, w.w_down, x2, io.out, false, T, d.H, d.F, scratch, p.scratch_bytes, s));
    TS_STEP(hook(TS_B_OUT_DENSE, io.out));
  } else {
    float* logits = reinterpret_cast<float*>(ws + p.logits);
    int32_t* tidx = reinterpret_cast<int32_t*>(ws + p.topk_idx);
    float* tw = reinterpret_cast<float*>(ws + p.topk_w);
    int32_t* counts = reinterpret_cast<int32_t*>(ws + p.counts);
    int32_t* offs = reinterpret_cast<int32_t*>(ws + p.offsets);
    int32_t* perm = reinterpret_cast<int32_t*>(ws + p.perm);
    int32_t* inv = reinterpret_cast<int32_t*>(ws + p.inv);
    ts_bf16* y = reinterpret_cast<ts_bf16*>(ws + p.y);
    const int rows = T * d.k;
    if (moe_router_supported(d.E, d.H))
      TS_STEP(launch_moe_router(h2, w.w_router, logits, T, d.E, d.H, s));
    else
      TS_STEP(launch_gemm(h2, w.w_router, nullptr, logits, true, T, d.E, d.H, scratch, p.scratch_bytes, s));
    TS_STEP(launch_moe_route(logits, T, d.E, d.k, tidx, tw, counts, offs, perm, s));
    pre(TS_B_GATE_UP);
    TS_STEP(launch_moe_gemm(h2, perm, d.k, w.w_gate_up, offs, gate_up, rows, d.E, 2 * d.F, d.H, s));
    TS_STEP(hook(TS_B_GATE_UP, gate_up));
    pre(TS_B_ACT);
    TS_STEP(launch_swiglu(gate_up, act, rows, d.F, s));
    TS_STEP(hook(TS_B_ACT, act));
    pre(TS_B_Y_MOE);
    TS_STEP(launch_moe_gemm(act, nullptr, 1, w.w_down, offs, y, rows, d.E, d.H, d.F, s));
    TS_STEP(hook(TS_B_Y_MOE, y));
    pre(TS_B_OUT_MOE);
    TS_STEP(launch_moe_combine(y, perm, tw, x2, io.out, inv, T, d.k, d.H, s));
    TS_STEP(hook(TS_B_OUT_MOE, io.out));
  }
#undef TS_STEP
  return TS_OK;
}

}  // namespace
}  // namespace ts

using namespace ts;

extern "C" {

const char* ts_strerror(int code) {
  switch (code) {
    case TS_OK: return "ok";
    case TS_ERR_INVALID_ARG: return "invalid argument";
    case TS_ERR_UNSUPPORTED_SHAPE: return "unsupported shape";
    case TS_ERR_WORKSPACE: return "workspace too small";
    case TS_ERR_HIP: return "HIP runtime error";
    default: return "unknown error";
  }
}
const char* ts_last_error(void) { return g_err; }
const char* ts_version(void) { return "tessera-mi355x 0.1 (gfx950)"; }

int ts_profile_begin(void** events, const char** names, int max_launches) {
  TS_REQUIRE(events != nullptr && names != nullptr && max_launches > 0, TS_ERR_INVALID_ARG,
             "ts_profile_begin: bad arguments");
  g_prof.events = reinterpret_cast<hipEvent_t*>(events);
  g_prof.names = names;
  g_prof.cap = max_launches;
  g_prof.used = 0;
  g_prof.active = true;
  return TS_OK;
}

int ts_profile_end(void) {
  const int n = g_prof.active ? g_prof.used : 0;
  g_prof = Profile();
  return n;
}

int ts_rmsnorm(const ts_bf16* x, const ts_bf16* gamma, ts_bf16* y, int T, int H, float eps, void* stream) {
  TS_REQUIRE(T >= 0 && H > 0, TS_ERR_INVALID_ARG, "ts_rmsnorm: T=%d H=%d", T, H);
  TS_REQUIRE(T == 0 || (x && gamma && y), TS_ERR_INVALID_ARG, "ts_rmsnorm: null pointer");
  TS_REQUIRE(aligned16(x) && aligned16(gamma) && aligned16(y), TS_ERR_INVALID_ARG, "ts_rmsnorm: pointer not 16-byte aligned");
  TS_REQUIRE(H % 8 == 0 && H <= 32768, TS_ERR_UNSUPPORTED_SHAPE, "ts_rmsnorm: H=%d must be a multiple of 8 and <= 32768", H);
  return launch_rmsnorm(x, gamma, y, T, H, eps, as_stream(stream));
}

static int check_gemm(const char* who, const void* A, const void* W, const void* C, int M, int N, int K) {
  TS_REQUIRE(M >= 0 && N > 0 && K > 0, TS_ERR_INVALID_ARG, "%s: M=%d N=%d K=%d", who, M, N, K);
  TS_REQUIRE(M == 0 || (A && W && C), TS_ERR_INVALID_ARG, "%s: null pointer", who);
  TS_REQUIRE(aligned16(A) && aligned16(W) && aligned16(C), TS_ERR_INVALID_ARG, "%s: pointer not 16-byte aligned", who);
  TS_REQUIRE(K % 8 == 0 && N % 2 == 0, TS_ERR_UNSUPPORTED_SHAPE, "%s: K=%d must be a multiple of 8 and N=%d even", who, K, N);
  return TS_OK;
}

size_t ts_gemm_workspace_bytes(int M, int N, int K) { return gemm_workspace_bytes(M, N, K); }

int ts_gemm_bf16(const ts_bf16* A, const ts_bf16* W, const ts_bf16* residual, ts_bf16* C, int M, int N, int K,
                 void* ws, size_t ws_bytes, void* stream) {
  int rc = check_gemm("ts_gemm_bf16", A, W, C, M, N, K);
  if (rc != TS_OK) return rc;
  TS_REQUIRE(aligned16(residual) && aligned16(ws), TS_ERR_INVALID_ARG, "ts_gemm_bf16: pointer not 16-byte aligned");
  return launch_gemm(A, W, residual, C, false, M, N, K, ws, ws_bytes, as_stream(stream));
}

int ts_gemm_bf16_f32out(const ts_bf16* A, const ts_bf16* W, float* C, int M, int N, int K, void* ws, size_t ws_bytes,
                        void* stream) {
  int rc = check_gemm("ts_gemm_bf16_f32out", A, W, C, M, N, K);
  if (rc != TS_OK) return rc;
  TS_REQUIRE(aligned16(ws), TS_ERR_INVALID_ARG, "ts_gemm_bf16_f32out: pointer not 16-byte aligned");
  return launch_gemm(A, W, nullptr, C, true, M, N, K, ws, ws_bytes, as_stream(stream));
}

int ts_rope(ts_bf16* q, ts_bf16* k, const ts_bf16* v, int q_stride, int kv_stride, const int32_t* pos,
            const int32_t* seq_id, const float* cos_sin, int table_len, ts_bf16* kcache, ts_bf16* vcache, int T, int nq,
            int nkv, int d, int Lcap, float base, void* stream) {
  TS_REQUIRE(T >= 0 && nq > 0 && nkv > 0 && d > 0, TS_ERR_INVALID_ARG, "ts_rope: T=%d nq=%d nkv=%d d=%d", T, nq, nkv, d);
  TS_REQUIRE(T == 0 || (q && k && pos), TS_ERR_INVALID_ARG, "ts_rope: null pointer");
  TS_REQUIRE((kcache == nullptr) == (vcache == nullptr), TS_ERR_INVALID_ARG, "ts_rope: kcache and vcache must both be set or both NULL");
  TS_REQUIRE(kcache == nullptr || (v && seq_id && Lcap > 0), TS_ERR_INVALID_ARG, "ts_rope: append needs v, seq_id and Lcap > 0");
  TS_REQUIRE(cos_sin == nullptr || table_len > 0, TS_ERR_INVALID_ARG, "ts_rope: table without length");
  TS_REQUIRE(base > 0.f, TS_ERR_INVALID_ARG, "ts_rope: base must be positive");
  TS_REQUIRE(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(cos_sin) && aligned16(kcache) && aligned16(vcache),
             TS_ERR_INVALID_ARG, "ts_rope: pointer not 16-byte aligned");
  TS_REQUIRE(d % 16 == 0 && d <= 256, TS_ERR_UNSUPPORTED_SHAPE, "ts_rope: d=%d must be a multiple of 16 and <= 256", d);
  TS_REQUIRE(q_stride % 8 == 0 && kv_stride % 8 == 0 && q_stride >= nq * d && kv_stride >= nkv * d,
             TS_ERR_UNSUPPORTED_SHAPE, "ts_rope: bad strides %d/%d", q_stride, kv_stride);
  return launch_rope(q, k, v, q_stride, kv_stride, pos, seq_id, cos_sin, cos_sin ? table_len : 0, kcache, vcache, T, nq,
                     nkv, d, Lcap, base, as_stream(stream));
}

int ts_rope_table(float* table_host, int table_len, int d, float base) {
  TS_REQUIRE(table_host != nullptr && table_len > 0 && d > 0 && d % 2 == 0 && base > 0.f, TS_ERR_INVALID_ARG,
             "ts_rope_table: bad arguments");
  const int half = d / 2;
  for (int p = 0; p < table_len; ++p) {
    float* row = table_host + (size_t)p * d;
    for (int i = 0; i < half; ++i) {
      const double theta = std::pow((double)base, -2.0 * (double)i / (double)d);
      const double ang = (double)p * theta;
      row[i] = (float)std::cos(ang);
      row[half + i] = (float)std::sin(ang);
    }
  }
  return TS_OK;
}

size_t ts_attention_decode_workspace_bytes(int B, int nq, int nkv, int d, int Lcap) {
  return attention_decode_workspace_bytes(B, nq, nkv, d, Lcap);
}

int ts_attention_decode(const ts_bf16* q, const ts_bf16* kcache, const ts_bf16* vcache, const int32_t* seq_lens,
                        ts_bf16* out, int B, int nq, int nkv, int d, int Lcap, float scale, void* ws, size_t ws_bytes,
                        void* stream) {
  TS_REQUIRE(B >= 0 && nq > 0 && nkv > 0 && d > 0 && Lcap > 0, TS_ERR_INVALID_ARG,
             "ts_attention_decode: B=%d nq=%d nkv=%d d=%d Lcap=%d", B, nq, nkv, d, Lcap);
  TS_REQUIRE(nq % nkv == 0, TS_ERR_INVALID_ARG, "ts_attention_decode: nq %% nkv != 0");
  TS_REQUIRE(B == 0 || (q && kcache && vcache && seq_lens && out), TS_ERR_INVALID_ARG, "ts_attention_decode: null pointer");
  TS_REQUIRE(aligned16(q) && aligned16(kcache) && aligned16(vcache) && aligned16(out) && aligned16(ws), TS_ERR_INVALID_ARG,
             "ts_attention_decode: pointer not 16-byte aligned");
  TS_REQUIRE(d == 64 || d == 128, TS_ERR_UNSUPPORTED_SHAPE, "ts_attention_decode: d=%d (64 or 128 supported)", d);
  TS_REQUIRE(nq / nkv <= 16, TS_ERR_UNSUPPORTED_SHAPE, "ts_attention_decode: GQA group %d > 16", nq / nkv);
  return launch_attention_decode(q, nq * d, kcache, vcache, seq_lens, out, B, nq, nkv, d, Lcap, scale, ws, ws_bytes,
                                 as_stream(stream));
}

int ts_attention_prefill(const ts_bf16* q, const ts_bf16* k, const ts_bf16* v, int q_stride, int kv_stride,
                         const int32_t* cu_seqlens, ts_bf16* out, int S, int T, int max_seqlen, int nq, int nkv, int d,
                         float scale, int causal, void* stream) {
  TS_REQUIRE(S >= 0 && T >= 0 && max_seqlen >= 0 && nq > 0 && nkv > 0 && d > 0, TS_ERR_INVALID_ARG,
             "ts_attention_prefill: S=%d T=%d nq=%d nkv=%d d=%d", S, T, nq, nkv, d);
  TS_REQUIRE(nq % nkv == 0, TS_ERR_INVALID_ARG, "ts_attention_prefill: nq %% nkv != 0");
  TS_REQUIRE(S == 0 || T == 0 || (q && k && v && cu_seqlens && out), TS_ERR_INVALID_ARG, "ts_attention_prefill: null pointer");
  TS_REQUIRE(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(out), TS_ERR_INVALID_ARG,
             "ts_attention_prefill: pointer not 16-byte aligned");
  TS_REQUIRE(d == 64 || d == 128, TS_ERR_UNSUPPORTED_SHAPE, "ts_attention_prefill: d=%d (64 or 128 supported)", d);
  TS_REQUIRE(q_stride % 8 == 0 && kv_stride % 8 == 0 && q_stride >= nq * d && kv_stride >= nkv * d,
             TS_ERR_UNSUPPORTED_SHAPE, "ts_attention_prefill: bad strides %d/%d", q_stride, kv_stride);
  return launch_attention_prefill(q, k, v, q_stride, kv_stride, cu_seqlens, out, S, T, max_seqlen, nq, nkv, d, scale,
                                  causal, as_stream(stream));
}

int ts_swiglu(const ts_bf16* gate_up, ts_bf16* out, int T, int F, void* stream) {
  TS_REQUIRE(T >= 0 && F > 0, TS_ERR_INVALID_ARG, "ts_swiglu: T=%d F=%d", T, F);
  TS_REQUIRE(T == 0 || (gate_up && out), TS_ERR_INVALID_ARG, "ts_swiglu: null pointer");
  TS_REQUIRE(aligned16(gate_up) && aligned16(out), TS_ERR_INVALID_ARG, "ts_swiglu: pointer not 16-byte aligned");
  TS_REQUIRE(F % 8 == 0, TS_ERR_UNSUPPORTED_SHAPE, "ts_swiglu: F=%d must be a multiple of 8", F);
  return launch_swiglu(gate_up, out, T, F, as_stream(stream));
}

int ts_moe_route(const float* logits, int T, int E, int k, int32_t* topk_idx, float* topk_w, int32_t* counts,
                 int32_t* offsets, int32_t* perm, void* stream) {
  TS_REQUIRE(T >= 0 && E > 0 && k >= 1 && k <= E, TS_ERR_INVALID_ARG, "ts_moe_route: T=%d E=%d k=%d", T, E, k);
  TS_REQUIRE(counts && offsets && (T == 0 || (logits && topk_idx && topk_w && perm)), TS_ERR_INVALID_ARG,
             "ts_moe_route: null pointer");
  TS_REQUIRE(E <= 64 && (long)T * k <= (1L << 20), TS_ERR_UNSUPPORTED_SHAPE, "ts_moe_route: E <= 64 and T*k <= 2^20 required");
  return launch_moe_route(logits, T, E, k, topk_idx, topk_w, counts, offsets, perm, as_stream(stream));
}

int ts_moe_gemm(const ts_bf16* A, const int32_t* row_map, int row_div, const ts_bf16* W, const int32_t* offsets,
                ts_bf16* C, int rows, int E, int N, int K, void* stream) {
  TS_REQUIRE(rows >= 0 && E > 0 && N > 0 && K > 0, TS_ERR_INVALID_ARG, "ts_moe_gemm: rows=%d E=%d N=%d K=%d", rows, E, N, K);
  TS_REQUIRE(rows == 0 || (A && W && offsets && C), TS_ERR_INVALID_ARG, "ts_moe_gemm: null pointer");
  TS_REQUIRE(row_map == nullptr || row_div >= 1, TS_ERR_INVALID_ARG, "ts_moe_gemm: row_div must be >= 1");
  TS_REQUIRE(aligned16(A) && aligned16(W) && aligned16(C), TS_ERR_INVALID_ARG, "ts_moe_gemm: pointer not 16-byte aligned");
  TS_REQUIRE(K % 8 == 0 && N % 2 == 0, TS_ERR_UNSUPPORTED_SHAPE, "ts_moe_gemm: K=%d must be a multiple of 8 and N=%d even", K, N);
  return launch_moe_gemm(A, row_map, row_map ? row_div : 1, W, offsets, C, rows, E, N, K, as_stream(stream));
}

int ts_moe_combine(const ts_bf16* y, const int32_t* perm, const float* topk_w, const ts_bf16* residual, ts_bf16* out,
                   int32_t* scratch_inv, int T, int k, int H, void* stream) {
  TS_REQUIRE(T >= 0 && k >= 1 && H > 0, TS_ERR_INVALID_ARG, "ts_moe_combine: T=%d k=%d H=%d", T, k, H);
  TS_REQUIRE(T == 0 || (y && perm && topk_w && out && scratch_inv), TS_ERR_INVALID_ARG, "ts_moe_combine: null pointer");
  TS_REQUIRE(aligned16(y) && aligned16(residual) && aligned16(out), TS_ERR_INVALID_ARG, "ts_moe_combine: pointer not 16-byte aligned");
  TS_REQUIRE(H % 8 == 0, TS_ERR_UNSUPPORTED_SHAPE, "ts_moe_combine: H=%d must be a multiple of 8", H);
  return launch_moe_combine(y, perm, topk_w, residual, out, scratch_inv, T, k, H, as_stream(stream));
}

// ---------------------------------------------------------------- layer
size_t ts_layer_workspace_bytes(const ts_layer_desc* desc, int T, int B) {
  if (validate_desc(desc, "ts_layer_workspace_bytes") != TS_OK || T < 0 || B < 0) return 0;
  return plan_layer(*desc, T, B).total;
}

int ts_layer_boundary(const ts_layer_desc* desc, int T, int B, int index, size_t* ws_offset, size_t* bytes) {
  int rc = validate_desc(desc, "ts_layer_boundary");
  if (rc != TS_OK) return rc;
  const int nb = desc->E > 0 ? TS_NB_MOE : TS_NB_DENSE;
  TS_REQUIRE(T >= 0 && B >= 0 && index >= 0 && index < nb && ws_offset && bytes, TS_ERR_INVALID_ARG,
             "ts_layer_boundary: bad index %d", index);
  LayerPlan p = plan_layer(*desc, T, B);
  *ws_offset = boundary_offset(p, *desc, index);
  *bytes = p.bytes[index];
  return TS_OK;
}

int ts_layer_moe_buffers(const ts_layer_desc* desc, int T, int B, size_t ws_offsets[6]) {
  int rc = validate_desc(desc, "ts_layer_moe_buffers");
  if (rc != TS_OK) return rc;
  TS_REQUIRE(desc->E > 0 && ws_offsets && T >= 0 && B >= 0, TS_ERR_INVALID_ARG, "ts_layer_moe_buffers: not a MoE layer");
  LayerPlan p = plan_layer(*desc, T, B);
  ws_offsets[0] = p.logits; ws_offsets[1] = p.topk_idx; ws_offsets[2] = p.topk_w;
  ws_offsets[3] = p.counts; ws_offsets[4] = p.offsets; ws_offsets[5] = p.perm;
  return TS_OK;
}

int ts_layer_node_accesses(const ts_layer_desc* desc, int T, int B, int kv_len, int node, ts_layer_access* out,
                           int max_accesses, int* n_accesses) {
  int rc = validate_desc(desc, "ts_layer_node_accesses");
  if (rc != TS_OK) return rc;
  const ts_layer_desc& d = *desc;
  const bool moe = d.E > 0;
  const int nb = moe ? TS_NB_MOE : TS_NB_DENSE;
  TS_REQUIRE(T >= 1 && B >= 1 && node >= 0 && node < nb && n_accesses != nullptr && max_accesses >= 0 &&
                 (out != nullptr || max_accesses == 0),
             TS_ERR_INVALID_ARG, "ts_layer_node_accesses: bad arguments (T=%d B=%d node=%d)", T, B, node);
  if (d.mode == TS_MODE_DECODE)
    TS_REQUIRE(T == B && kv_len >= 1 && kv_len <= d.Lcap, TS_ERR_INVALID_ARG,
               "ts_layer_node_accesses: decode needs T == B and 1 <= kv_len <= Lcap");
  const LayerPlan p = plan_layer(d, T, B);
  std::vector<ts_layer_access> acc;
  auto add = [&](int buffer, int kind, uint64_t off, uint64_t extent, uint64_t bytes, int64_t adv = 0) {
    if (extent == 0) return;
    acc.push_back(ts_layer_access{buffer, kind, off, extent, bytes, adv});
  };
  auto full = [&](int buffer, int kind, uint64_t off, uint64_t n) { add(buffer, kind, off, n, n); };
  // boundary i as the node that produces it writes it and as later nodes read it
  auto bnd = [&](int kind, int i) {
    if (i == nb - 1) full(TS_BUF_OUT, kind, 0, p.bytes[i]);
    else full(TS_BUF_WORKSPACE, kind, boundary_offset(p, d, i), p.bytes[i]);
  };
  auto scratch = [&](size_t bytes) { full(TS_BUF_WORKSPACE, TS_ACC_PRIVATE, p.scratch, bytes); };
  const uint64_t xbytes = (uint64_t)T * d.H * 2, row = (uint64_t)d.d * 2;
  const uint64_t nqd = (uint64_t)d.nq * d.d, nqkv = (uint64_t)(d.nq + 2 * d.nkv) * d.d;
  const uint64_t cache_bytes = (uint64_t)B * d.nkv * d.Lcap * row;
  const int rows = moe ? T * d.k : T;
  switch (node) {
    case TS_B_H1:
      full(TS_BUF_X, TS_ACC_READ, 0, xbytes);
      bnd(TS_ACC_WRITE, TS_B_H1);
      // the first kernel of the layer also zeroes the arrival counters of the attention kernel
      full(TS_BUF_WORKSPACE, TS_ACC_PRIVATE, p.counters, (uint64_t)p.counter_words * 4);
      break;
    case TS_B_QKV:
      bnd(TS_ACC_READ, TS_B_H1);
      bnd(TS_ACC_WRITE, TS_B_QKV);
      scratch(gemm_workspace_bytes(T, (int)nqkv, d.H));
      if (d.mode == TS_MODE_DECODE) {   // one new row per (sequence, kv head), one position further every iteration
        for (int b = 0; b < B; ++b)
          for (int h = 0; h < d.nkv; ++h) {
            const uint64_t o = (((uint64_t)b * d.nkv + h) * d.Lcap + (uint64_t)(kv_len - 1)) * row;
            add(TS_BUF_KCACHE, TS_ACC_WRITE, o, row, row, (int64_t)row);
            add(TS_BUF_VCACHE, TS_ACC_WRITE, o, row, row, (int64_t)row);
          }
      } else {
        const uint64_t kv_new = std::min<uint64_t>((uint64_t)T * d.nkv * row, cache_bytes);
        add(TS_BUF_KCACHE, TS_ACC_WRITE, 0, cache_bytes, kv_new);
        add(TS_BUF_VCACHE, TS_ACC_WRITE, 0, cache_bytes, kv_new);
      }
      break;
    case TS_B_ATTN:
      if (d.mode == TS_MODE_DECODE) {
        add(TS_BUF_WORKSPACE, TS_ACC_READ, p.qkv, p.bytes[TS_B_QKV], (uint64_t)T * nqd * 2);   // the q columns
        const uint64_t kv_read = (uint64_t)B * d.nkv * kv_len * row;
        add(TS_BUF_KCACHE, TS_ACC_READ, 0, cache_bytes, kv_read);
        add(TS_BUF_VCACHE, TS_ACC_READ, 0, cache_bytes, kv_read);
        scratch(attention_decode_workspace_bytes(B, d.nq, d.nkv, d.d, d.Lcap));
        full(TS_BUF_WORKSPACE, TS_ACC_PRIVATE, p.counters, (uint64_t)p.counter_words * 4);
      } else {
        bnd(TS_ACC_READ, TS_B_QKV);
      }
      bnd(TS_ACC_WRITE, TS_B_ATTN);
      break;
    case TS_B_X2:
      bnd(TS_ACC_READ, TS_B_ATTN);
      full(TS_BUF_X, TS_ACC_READ, 0, xbytes);
      bnd(TS_ACC_WRITE, TS_B_X2);
      scratch(gemm_workspace_bytes(T, d.H, d.nq * d.d));
      break;
    case TS_B_H2:
      bnd(TS_ACC_READ, TS_B_X2);
      bnd(TS_ACC_WRITE, TS_B_H2);
      break;
    case TS_B_GATE_UP:
      bnd(TS_ACC_READ, TS_B_H2);
      bnd(TS_ACC_WRITE, TS_B_GATE_UP);
      if (!moe) {
        scratch(gemm_workspace_bytes(T, 2 * d.F, d.H));
        if (gemm_mfma256_glu_supported(T, d.F, d.H)) bnd(TS_ACC_WRITE, TS_B_ACT);   // activation in the epilogue
      } else {   // router, routing and the grouped projection: the routing tables are this node's side outputs
        full(TS_BUF_WORKSPACE, TS_ACC_WRITE, p.logits, (uint64_t)T * d.E * 4);
        full(TS_BUF_WORKSPACE, TS_ACC_WRITE, p.topk_idx, (uint64_t)T * d.k * 4);
        full(TS_BUF_WORKSPACE, TS_ACC_WRITE, p.topk_w, (uint64_t)T * d.k * 4);
        full(TS_BUF_WORKSPACE, TS_ACC_WRITE, p.counts, (uint64_t)d.E * 4);
        full(TS_BUF_WORKSPACE, TS_ACC_WRITE, p.offsets, (uint64_t)(d.E + 1) * 4);
        full(TS_BUF_WORKSPACE, TS_ACC_WRITE, p.perm, (uint64_t)T * d.k * 4);
        if (!moe_router_supported(d.E, d.H)) scratch(gemm_workspace_bytes(T, d.E, d.H));
      }
      break;
    case TS_B_ACT:
      bnd(TS_ACC_READ, TS_B_GATE_UP);
      bnd(TS_ACC_WRITE, TS_B_ACT);
      break;
    default:
      if (!moe) {   // TS_B_OUT_DENSE
        bnd(TS_ACC_READ, TS_B_ACT);
        bnd(TS_ACC_READ, TS_B_X2);
        bnd(TS_ACC_WRITE, TS_B_OUT_DENSE);
        scratch(gemm_workspace_bytes(T, d.H, d.F));
      } else if (node == TS_B_Y_MOE) {
        bnd(TS_ACC_READ, TS_B_ACT);
        full(TS_BUF_WORKSPACE, TS_ACC_READ, p.offsets, (uint64_t)(d.E + 1) * 4);
        bnd(TS_ACC_WRITE, TS_B_Y_MOE);
      } else {   // TS_B_OUT_MOE
        bnd(TS_ACC_READ, TS_B_Y_MOE);
        bnd(TS_ACC_READ, TS_B_X2);
        full(TS_BUF_WORKSPACE, TS_ACC_READ, p.perm, (uint64_t)rows * 4);
        full(TS_BUF_WORKSPACE, TS_ACC_READ, p.topk_w, (uint64_t)rows * 4);
        full(TS_BUF_WORKSPACE, TS_ACC_PRIVATE, p.inv, (uint64_t)rows * 4);
        bnd(TS_ACC_WRITE, TS_B_OUT_MOE);
      }
      break;
  }
  *n_accesses = (int)acc.size();
  TS_REQUIRE((int)acc.size() <= max_accesses, TS_ERR_WORKSPACE, "ts_layer_node_accesses: %zu accesses, room for %d", acc.size(),
             max_accesses);
  std::copy(acc.begin(), acc.end(), out);
  return TS_OK;
}

int ts_layer_forward(const ts_layer_desc* desc, const ts_layer_weights* w, const ts_layer_io* io, void* ws,
                     size_t ws_bytes, void* stream) {
  int rc = validate_desc(desc, "ts_layer_forward");
  if (rc != TS_OK) return rc;
  rc = validate_io(desc, w, io, "ts_layer_forward");
  if (rc != TS_OK) return rc;
  const size_t need = plan_layer(*desc, io->T, io->B).total;
  TS_REQUIRE(io->T == 0 || (ws != nullptr && ws_bytes >= need), TS_ERR_WORKSPACE,
             "ts_layer_forward: workspace %zu bytes < required %zu", ws_bytes, need);
  TS_REQUIRE(aligned16(ws), TS_ERR_INVALID_ARG, "ts_layer_forward: workspace not 16-byte aligned");
  return layer_forward_impl(*desc, *w, *io, reinterpret_cast<char*>(ws), as_stream(stream), [](int) {},
                            [](int, const void*) { return TS_OK; });
}

// ---------------------------------------------------------------- pipeline
struct ts_pipeline {
  ts_layer_desc desc;
  int max_mb;
  bool events_ready = false;            // events are created by the first step (creation itself needs no GPU)
  std::vector<hipEvent_t> boundary_ev;  // [max_mb][TS_NB_MOE]
  std::vector<hipEvent_t> packed_ev;    // [max_mb]
  std::vector<hipEvent_t> kv_ready_ev;  // [max_mb] compute stream: K/V rows of the step are in the projection buffer
  std::vector<hipEvent_t> kv_sent_ev;   // [max_mb] delta stream: rows have left
  // [2][max_mb] compute stream: the micro-batch's last kernel has been enqueued.  Two sets used by alternate
  // steps, so that a step can wait for the previous step's events after it has recorded some of its own.
  std::vector<hipEvent_t> done_ev;
  int parity = 0;
  // background replication of the rows appended to the KV cache (off while delta_stream is null)
  hipStream_t delta_stream = nullptr;
  char* delta_dev = nullptr;
  char* delta_host = nullptr;
  size_t delta_bytes = 0;
  bool delta_on = false;
  // what the previous step left in flight, per workspace slot (-1: nothing): the last micro-batch whose boundary
  // sends / KV rows / kernels used the slot, the compute stream it ran on, and the slot geometry of that step
  // (a step with another geometry waits for all of it)
  std::vector<int> prev_packed, prev_kv_sent, prev_done;   // [max_mb]
  std::vector<hipStream_t> prev_stream;                    // [max_mb]
  size_t prev_slot_bytes = 0;
  int prev_nslot = 0;
  const void* prev_ws = nullptr;
  int link_slowdown = 1;   // every boundary tensor crosses the host link this many times
};

static int pipeline_ensure_events(ts_pipeline* p) {
  if (p->events_ready) return TS_OK;
  const int m = p->max_mb;
  const int nbe = m * TS_NB_MOE;
  const int n = nbe + 5 * m;
  for (int i = 0; i < n; ++i) {
    hipEvent_t e;
    TS_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming | hipEventReleaseToDevice));
    if (i < nbe) p->boundary_ev.push_back(e);
    else if (i < nbe + m) p->packed_ev.push_back(e);
    else if (i < nbe + 2 * m) p->kv_ready_ev.push_back(e);
    else if (i < nbe + 3 * m) p->kv_sent_ev.push_back(e);
    else p->done_ev.push_back(e);
  }
  p->events_ready = true;
  return TS_OK;
}

int ts_pipeline_create(const ts_layer_desc* desc, int max_micro_batches, ts_pipeline** out) {
  int rc = validate_desc(desc, "ts_pipeline_create");
  if (rc != TS_OK) return rc;
  TS_REQUIRE(out != nullptr && max_micro_batches > 0 && max_micro_batches <= 64, TS_ERR_INVALID_ARG,
             "ts_pipeline_create: bad arguments");
  ts_pipeline* p = new (std::nothrow) ts_pipeline();
  TS_REQUIRE(p != nullptr, TS_ERR_INVALID_ARG, "ts_pipeline_create: out of host memory");
  p->desc = *desc;
  p->max_mb = max_micro_batches;
  p->prev_packed.assign(max_micro_batches, -1);
  p->prev_kv_sent.assign(max_micro_batches, -1);
  p->prev_done.assign(max_micro_batches, -1);
  p->prev_stream.assign(max_micro_batches, nullptr);
  *out = p;
  return TS_OK;
}

void ts_pipeline_destroy(ts_pipeline* p) {
  if (p == nullptr) return;
  for (hipEvent_t e : p->boundary_ev) (void)hipEventDestroy(e);
  for (hipEvent_t e : p->packed_ev) (void)hipEventDestroy(e);
  for (hipEvent_t e : p->kv_ready_ev) (void)hipEventDestroy(e);
  for (hipEvent_t e : p->kv_sent_ev) (void)hipEventDestroy(e);
  for (hipEvent_t e : p->done_ev) (void)hipEventDestroy(e);
  delete p;
}

size_t ts_pipeline_workspace_slot_bytes(const ts_layer_desc* desc, const int32_t* Ts, const int32_t* Bs, int n_mb) {
  if (desc == nullptr || Ts == nullptr || Bs == nullptr || n_mb <= 0) return 0;
  if (validate_desc(desc, "ts_pipeline_workspace_slot_bytes") != TS_OK) return 0;
  size_t slot = 0;
  for (int i = 0; i < n_mb; ++i) {
    if (Ts[i] < 0 || Bs[i] < 0) return 0;
    slot = std::max(slot, round_up(plan_layer(*desc, Ts[i], Bs[i]).total, 256));
  }
  return slot;
}

size_t ts_pipeline_kv_delta_stride(const ts_layer_desc* desc, int T) {
  if (desc == nullptr || T < 0 || validate_desc(desc, "ts_pipeline_kv_delta_stride") != TS_OK) return 0;
  return round_up((size_t)T * 2 * desc->nkv * desc->d * sizeof(ts_bf16), 256);
}

int ts_pipeline_set_kv_delta(ts_pipeline* p, void* delta_stream, void* dev_slots, void* host_slots, size_t bytes) {
  TS_REQUIRE(p != nullptr, TS_ERR_INVALID_ARG, "ts_pipeline_set_kv_delta: null pipeline");
  if (dev_slots == nullptr && host_slots == nullptr) {
    p->delta_on = false;
    return TS_OK;
  }
  TS_REQUIRE(dev_slots != nullptr && host_slots != nullptr && aligned16(dev_slots) && aligned16(host_slots), TS_ERR_INVALID_ARG,
             "ts_pipeline_set_kv_delta: both slot buffers are needed, 16-byte aligned");
  p->delta_stream = as_stream(delta_stream);
  p->delta_dev = reinterpret_cast<char*>(dev_slots);
  p->delta_host = reinterpret_cast<char*>(host_slots);
  p->delta_bytes = bytes;
  p->delta_on = true;
  return TS_OK;
}

int ts_pipeline_boundary_layout(const ts_layer_desc* desc, int T, int B, uint64_t boundary_mask, size_t* offsets,
                                int* n_boundaries) {
  int rc = validate_desc(desc, "ts_pipeline_boundary_layout");
  if (rc != TS_OK) return rc;
  TS_REQUIRE(offsets && n_boundaries && T >= 0 && B >= 0, TS_ERR_INVALID_ARG, "ts_pipeline_boundary_layout: bad arguments");
  const int nb = desc->E > 0 ? TS_NB_MOE : TS_NB_DENSE;
  LayerPlan p = plan_layer(*desc, T, B);
  size_t off = 0;
  int n = 0;
  for (int i = 0; i < nb; ++i) {
    if (!((boundary_mask >> i) & 1)) continue;
    offsets[n++] = off;
    off += round_up(p.bytes[i], 16);
  }
  offsets[n] = off;
  *n_boundaries = n;
  return TS_OK;
}

size_t ts_pipeline_slot_stride(const ts_layer_desc* desc, int T, int B, uint64_t boundary_mask) {
  size_t offs[TS_NB_MOE + 1];
  int n = 0;
  if (ts_pipeline_boundary_layout(desc, T, B, boundary_mask, offs, &n) != TS_OK) return 0;
  return round_up(offs[n], 256);
}

int ts_pipeline_set_link_slowdown(ts_pipeline* p, int factor) {
  TS_REQUIRE(p != nullptr, TS_ERR_INVALID_ARG, "ts_pipeline_set_link_slowdown: null pipeline");
  TS_REQUIRE(factor >= 1 && factor <= 64, TS_ERR_INVALID_ARG, "ts_pipeline_set_link_slowdown: factor %d outside [1,64]",
             factor);
  p->link_slowdown = factor;
  return TS_OK;
}

int ts_pipeline_step(ts_pipeline* p, const ts_layer_weights* w, const ts_layer_io* mb, int n_mb,
                     void* compute_streams[2], void* copy_stream, uint64_t boundary_mask, int copy_mode,
                     void* dev_staging, void* pinned_host, size_t staging_bytes, void* ws, size_t ws_bytes) {
  TS_REQUIRE(p != nullptr && w != nullptr && mb != nullptr && compute_streams != nullptr, TS_ERR_INVALID_ARG,
             "ts_pipeline_step: null argument");
  TS_REQUIRE(n_mb >= 1 && n_mb <= p->max_mb, TS_ERR_INVALID_ARG, "ts_pipeline_step: n_mb=%d outside [1,%d]", n_mb, p->max_mb);
  TS_REQUIRE(copy_mode >= TS_PIPE_COPY_SIDE_STREAM && copy_mode <= TS_PIPE_COPY_COALESCED_HALVES,
             TS_ERR_INVALID_ARG, "ts_pipeline_step: unknown copy mode %d", copy_mode);
  const ts_layer_desc& d = p->desc;
  const int nb = d.E > 0 ? TS_NB_MOE : TS_NB_DENSE;
  if (nb < 64) boundary_mask &= ((1ull << nb) - 1ull);
  int Tmax = 0, Bmax = 0;
  for (int i = 0; i < n_mb; ++i) {
    int rc = validate_io(&d, w, &mb[i], "ts_pipeline_step");
    if (rc != TS_OK) return rc;
    if (mb[i].T > Tmax) Tmax = mb[i].T;
    if (mb[i].B > Bmax) Bmax = mb[i].B;
  }
  // A micro-batch lays its workspace slot out with the plan of its own (T, B), and that size is not monotone in
  // T or B (the split-K and split-KV plans change form with the row count), so the slot is the largest plan
  // over the micro-batches, not the plan of the largest micro-batch.
  size_t slot_bytes = 0;
  for (int i = 0; i < n_mb; ++i) slot_bytes = std::max(slot_bytes, round_up(plan_layer(d, mb[i].T, mb[i].B).total, 256));
  TS_REQUIRE(ws != nullptr && ws_bytes >= 2 * slot_bytes, TS_ERR_WORKSPACE,
             "ts_pipeline_step: workspace %zu bytes < required %zu (two slots of ts_pipeline_workspace_slot_bytes)",
             ws_bytes, 2 * slot_bytes);
  const size_t stride = ts_pipeline_slot_stride(&d, Tmax, Bmax, boundary_mask);
  TS_REQUIRE(boundary_mask == 0 || (dev_staging && pinned_host && staging_bytes >= stride * (size_t)n_mb),
             TS_ERR_WORKSPACE, "ts_pipeline_step: staging %zu bytes < required %zu", staging_bytes, stride * (size_t)n_mb);
  TS_REQUIRE(aligned16(ws) && aligned16(dev_staging) && aligned16(pinned_host), TS_ERR_INVALID_ARG,
             "ts_pipeline_step: buffer not 16-byte aligned");
  hipStream_t cs[2] = {as_stream(compute_streams[0]), as_stream(compute_streams[1])};
  hipStream_t copy = as_stream(copy_stream);
  const size_t dstride = ts_pipeline_kv_delta_stride(&d, Tmax);
  TS_REQUIRE(!p->delta_on || p->delta_bytes >= dstride * (size_t)n_mb, TS_ERR_WORKSPACE,
             "ts_pipeline_step: KV delta slots %zu bytes < required %zu", p->delta_bytes, dstride * (size_t)n_mb);
  {
    int rc = pipeline_ensure_events(p);
    if (rc != TS_OK) return rc;
  }

  // Micro-batch i works in workspace slot i % nslot, with as many slots as the workspace holds (two at least):
  // with a slot of its own a micro-batch never waits for the transfers of an earlier one of the same step
  // (with two slots every micro-batch from the third on starts only after the last send of the one two before
  // it, which cannot begin before that one's last kernel).
  const int nslot = (int)std::min<size_t>((size_t)n_mb, std::max<size_t>(2, ws_bytes / slot_bytes));
  const bool same_geometry = p->prev_nslot == nslot && p->prev_slot_bytes == slot_bytes && p->prev_ws == ws;
  const bool sends = boundary_mask != 0 && copy_mode != TS_PIPE_COPY_SERIALISED;
  hipEvent_t* done_now = p->done_ev.data() + (size_t)p->parity * p->max_mb;
  hipEvent_t* done_prev = p->done_ev.data() + (size_t)(p->parity ^ 1) * p->max_mb;
  // Steps may follow each other without a host synchronisation.  What the previous step left in flight in slot h:
  // the sends that read it, and the kernels of its last user when those ran on another stream.
  auto wait_prev_slot = [&](hipStream_t s, int h) -> int {
    if (p->prev_packed[h] >= 0) TS_HIP(hipStreamWaitEvent(s, p->packed_ev[p->prev_packed[h]], 0));
    if (p->prev_kv_sent[h] >= 0) TS_HIP(hipStreamWaitEvent(s, p->kv_sent_ev[p->prev_kv_sent[h]], 0));
    if (p->prev_done[h] >= 0 && p->prev_stream[h] != s) TS_HIP(hipStreamWaitEvent(s, done_prev[p->prev_done[h]], 0));
    return TS_OK;
  };
  if (!same_geometry) {   // other slots than last time: both streams wait for all of it, before this step records anything
    for (int c = 0; c < (n_mb > 1 ? 2 : 1); ++c)
      for (int h = 0; h < p->prev_nslot; ++h) {
        int rc = wait_prev_slot(cs[c], h);
        if (rc != TS_OK) return rc;
      }
  }
  for (int i = 0; i < n_mb; ++i) {
    hipStream_t s = cs[i & 1];
    char* wsh = reinterpret_cast<char*>(ws) + (size_t)(i % nslot) * slot_bytes;
    // A slot is reused by every nslot-th micro-batch.  Its next user waits (a) until the side streams have read
    // what they send from it and (b), when it runs on the other compute stream (odd nslot), until the previous
    // user's kernels are done: the sends cover only the kernels up to the last flagged boundary.
    if (i >= nslot) {
      if (sends) TS_HIP(hipStreamWaitEvent(s, p->packed_ev[i - nslot], 0));
      if (p->delta_on) TS_HIP(hipStreamWaitEvent(s, p->kv_sent_ev[i - nslot], 0));   // its rows sit in that slot
      if (cs[(i - nslot) & 1] != s) TS_HIP(hipStreamWaitEvent(s, done_now[i - nslot], 0));
    } else if (same_geometry && i < p->prev_nslot) {   // same slots as last time: only this slot's last user matters
      int rc = wait_prev_slot(s, i);
      if (rc != TS_OK) return rc;
    }
    const LayerPlan plan = plan_layer(d, mb[i].T, mb[i].B);
    size_t offs[TS_NB_MOE + 1];
    int n = 0;
    int rc = ts_pipeline_boundary_layout(&d, mb[i].T, mb[i].B, boundary_mask, offs, &n);
    if (rc != TS_OK) return rc;
    char* slot_dev = reinterpret_cast<char*>(dev_staging) + (size_t)i * stride;
    char* slot_host = reinterpret_cast<char*>(pinned_host) + (size_t)i * stride;
    int ordinal = 0;
    CopySegments pending{};
    const bool halves = copy_mode == TS_PIPE_COPY_COALESCED_HALVES;
    const bool coalesce = copy_mode == TS_PIPE_COPY_COALESCED || halves;
    const bool serial = copy_mode == TS_PIPE_COPY_SERIALISED;
    // where coalesced sends leave: the designated boundaries and the end of the layer
    auto send_point = [&](int index) {
      if (halves) return index == TS_B_X2 || index == nb - 1;
      return index == TS_B_QKV || index == TS_B_H2 || index == TS_B_ACT || index == nb - 1;
    };
    // Before the launch function that completes boundary `index`: if a send will follow it, let its last
    // kernel carry the boundary's event (fires when the kernel completes; no marker packet on the compute
    // stream).  `attached` tells the hook whether a kernel took it.
    bool armed = false, attached = false;
    auto pre = [&](int index) {
      const bool flagged = (boundary_mask >> index) & 1;
      armed = !serial && (coalesce ? send_point(index) && (flagged || pending.n > 0) : flagged);
      if (armed) arm_stop_event(p->boundary_ev[(size_t)i * TS_NB_MOE + index]);
    };
    // send what is pending: the boundary's event (carried by its kernel, else recorded here), one pack launch
    // on the copy stream
    auto flush = [&](int index) -> int {
      if (pending.n == 0) return TS_OK;
      hipEvent_t e = p->boundary_ev[(size_t)i * TS_NB_MOE + index];
      if (!attached) TS_HIP(hipEventRecord(e, s));
      TS_HIP(hipStreamWaitEvent(copy, e, 0));
      int rc2 = launch_copy16_multi(pending, slot_dev, slot_host, copy, p->link_slowdown);
      pending.n = 0;
      return rc2;
    };
    auto hook = [&](int index, const void* ptr) -> int {
      attached = armed && !disarm_stop_event();   // armed and no longer pending: a kernel carries the event
      if (!armed) disarm_stop_event();
      armed = false;
      if (index == TS_B_QKV && p->delta_on) {
        // the K and V rows this step appends to the cache are columns [nq d, (nq + 2 nkv) d) of the projection
        // buffer: one strided pack on the delta stream, behind the boundary's own event if the RoPE kernel
        // carries it, else behind an event recorded here
        hipEvent_t ready = attached ? p->boundary_ev[(size_t)i * TS_NB_MOE + index] : p->kv_ready_ev[i];
        if (!attached) TS_HIP(hipEventRecord(ready, s));
        TS_HIP(hipStreamWaitEvent(p->delta_stream, ready, 0));
        const int nqkv = (d.nq + 2 * d.nkv) * d.d;
        int rc2 = launch_copy_rows(reinterpret_cast<const ts_bf16*>(ptr) + (size_t)d.nq * d.d, (size_t)nqkv * sizeof(ts_bf16),
                                   (size_t)2 * d.nkv * d.d * sizeof(ts_bf16), mb[i].T, p->delta_dev + (size_t)i * dstride,
                                   p->delta_host + (size_t)i * dstride, p->delta_stream);
        if (rc2 != TS_OK) return rc2;
        TS_HIP(hipEventRecord(p->kv_sent_ev[i], p->delta_stream));
      }
      const bool flagged = (boundary_mask >> index) & 1;
      if (flagged) {
        const size_t bytes = round_up(plan.bytes[index], 16);
        const size_t o = offs[ordinal++];
        if (coalesce) {
          pending.src[pending.n] = ptr;
          pending.dst_off16[pending.n] = o / 16;
          pending.n16[pending.n] = bytes / 16;
          ++pending.n;
        } else {
          hipStream_t target = s;
          if (!serial) {
            hipEvent_t e = p->boundary_ev[(size_t)i * TS_NB_MOE + index];
            if (!attached) TS_HIP(hipEventRecord(e, s));
            TS_HIP(hipStreamWaitEvent(copy, e, 0));
            target = copy;
          }
          // one kernel packs the tensor into the device slot and stores it to the pinned host slot
          return launch_copy16(ptr, slot_dev + o, bytes, target, slot_host + o, p->link_slowdown);
        }
      }
      // coalesced sends leave after RoPE, after the second norm, after SwiGLU and at the end of the layer (the
      // last one is then only the layer output: the next user of this workspace slot waits for it)
      // (TS_PIPE_COPY_COALESCED_HALVES: after the attention half of the layer and at the end)
      if (coalesce && (send_point(index) || pending.n == 4)) return flush(index);
      return TS_OK;
    };
    rc = layer_forward_impl(d, *w, mb[i], wsh, s, pre, hook);
    disarm_stop_event();
    if (rc != TS_OK) return rc;
    if (sends) TS_HIP(hipEventRecord(p->packed_ev[i], copy));
    // the slot's next user may run on the other compute stream (in this step when nslot is odd; in the next
    // step whenever the caller passes other streams or another workspace): mark the end of this one's kernels
    const bool last_user = i + nslot >= n_mb;
    if (last_user || cs[(i + nslot) & 1] != s) TS_HIP(hipEventRecord(done_now[i], s));
  }
  for (int h = 0; h < nslot; ++h) {
    int last = -1;   // last micro-batch that used slot h
    for (int i = h; i < n_mb; i += nslot) last = i;
    p->prev_packed[h] = (last >= 0 && sends) ? last : -1;
    p->prev_kv_sent[h] = (last >= 0 && p->delta_on) ? last : -1;
    p->prev_done[h] = last;
    p->prev_stream[h] = last >= 0 ? cs[last & 1] : nullptr;
  }
  p->prev_nslot = nslot;
  p->prev_slot_bytes = slot_bytes;
  p->prev_ws = ws;
  p->parity ^= 1;
  return TS_OK;
}

}  // extern "C"
