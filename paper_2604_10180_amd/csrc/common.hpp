// Shared device/host helpers for the gfx950 decoder-layer kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/tessera.h"

namespace ts {

// ---- error plumbing (host) -------------------------------------------------
void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);
int check_hip(hipError_t e, const char* what);

#define TS_REQUIRE(cond, code, ...)            \
  do {                                         \
    if (!(cond)) return ::ts::fail((code), __VA_ARGS__); \
  } while (0)

#define TS_HIP(expr)                                         \
  do {                                                       \
    int _rc = ::ts::check_hip((expr), #expr);                \
    if (_rc != TS_OK) return _rc;                            \
  } while (0)

// checks the launch that was just issued
#define TS_LAUNCH_CHECK(name) TS_HIP(hipGetLastError())

// Optional per-launch timing: when a profile is active on the calling thread, every kernel
// launch is bracketed by two caller-supplied events recorded on the launch stream.
void prof_begin(const char* name, hipStream_t s);
void prof_end(hipStream_t s);

// A caller (the pipelined step) can arm an event on its thread that the last kernel of the next launch function
// carries as its stop event: the event then fires when that kernel completes and costs the stream no marker
// packet of its own (a separate hipEventRecord between two kernels measured 1.4 us more per occurrence).  Only
// launches written as TS_LAUNCH_LAST take the armed event, and a launch function uses that form for the final
// kernel it enqueues and for no other, so an event can never fire before the function's result is complete;
// a path that does not take it leaves it armed, and the caller falls back to recording it.
void arm_stop_event(hipEvent_t e);
hipEvent_t take_stop_event();    // the armed event (then disarmed), or nullptr
bool disarm_stop_event();        // true if an event was still armed

#define TS_LAUNCH_EX(last, name, kernel, grid, block, smem, stream, ...)                              \
  do {                                                                                                \
    ::ts::prof_begin(name, stream);                                                                   \
    hipEvent_t ts_stop_ev_ = (last) ? ::ts::take_stop_event() : nullptr;                              \
    if (ts_stop_ev_ != nullptr)                                                                       \
      hipExtLaunchKernelGGL(kernel, grid, block, smem, stream, nullptr, ts_stop_ev_, 0, __VA_ARGS__);  \
    else                                                                                              \
      hipLaunchKernelGGL(kernel, grid, block, smem, stream, __VA_ARGS__);                             \
    ::ts::prof_end(stream);                                                                           \
  } while (0)
#define TS_LAUNCH(name, kernel, grid, block, smem, stream, ...) \
  TS_LAUNCH_EX(false, name, kernel, grid, block, smem, stream, __VA_ARGS__)
#define TS_LAUNCH_LAST(name, kernel, grid, block, smem, stream, ...) \
  TS_LAUNCH_EX(true, name, kernel, grid, block, smem, stream, __VA_ARGS__)

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// ---- device vector types ----------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

union U4 {
  uint4 u;
  bf16x8 b;
  uint32_t w[4];
  uint16_t h[8];
};

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf_to_f(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// two floats -> packed bf16 pair (round to nearest even; hardware v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ uint16_t f_to_bf(float f) {
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}

__device__ __forceinline__ uint4 ldg16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
// 16-byte load of data that is read once (cache streams, weight streams): the non-temporal hint keeps it from
// displacing what other kernels and workgroups re-read, and a pure read stream measures 7.0 TB/s with it
// against 6.3 TB/s without.
__device__ __forceinline__ uint4 ldg16_stream(const void* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}
// Predicated 16-byte load without a branch: `p` must be a readable address even when !ok
// (callers clamp it); the result is zeroed when !ok.  (A conditional expression around a
// 16-byte load is split by the compiler into four branchy 4-byte loads.)
__device__ __forceinline__ uint4 ldg16_or_zero(const void* p, bool ok) {
  uint4 v = *reinterpret_cast<const uint4*>(p);
  v.x = ok ? v.x : 0u; v.y = ok ? v.y : 0u; v.z = ok ? v.z : 0u; v.w = ok ? v.w : 0u;
  return v;
}
__device__ __forceinline__ void stg16(void* p, uint4 v) { *reinterpret_cast<uint4*>(p) = v; }

// Device-coherent 8-byte accesses (relaxed atomics at agent scope: they go through to the
// memory side instead of staying in one XCD's L2).  Used for the partial results that one
// workgroup writes and a workgroup on another XCD reads within the same launch; they avoid the
// whole-L2 write-back / invalidate that an agent-scope fence costs.
__device__ __forceinline__ void st_dev_f32x2(float* p, float a, float b) {
  const uint64_t v = ((uint64_t)__float_as_uint(b) << 32) | __float_as_uint(a);
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ f32x2 ld_dev_f32x2(const float* p) {
  const uint64_t v = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  f32x2 r = {__uint_as_float((uint32_t)v), __uint_as_float((uint32_t)(v >> 32))};
  return r;
}
__device__ __forceinline__ void st_dev_f32(float* p, float a) {
  __hip_atomic_store(p, a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev_f32(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// all of this wave's stores have been acknowledged (then a barrier covers the workgroup)
__device__ __forceinline__ void wait_stores() { __builtin_amdgcn_s_waitcnt(0x0F70); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- internal launchers (host), one per kernel family -----------------------
// `zero`/`nzero`: optional int32 words the kernel clears on the side (the layer uses this to arm
// the arrival counters of the kernels that follow on the same stream).
int launch_rmsnorm(const ts_bf16* x, const ts_bf16* gamma, ts_bf16* y, int T, int H, float eps, hipStream_t s,
                   int32_t* zero = nullptr, int nzero = 0);
int launch_swiglu(const ts_bf16* gu, ts_bf16* out, int T, int F, hipStream_t s);
int launch_rope(ts_bf16* q, ts_bf16* k, const ts_bf16* v, int q_stride, int kv_stride, const int32_t* pos,
                const int32_t* seq_id, const float* cos_sin, int table_len, ts_bf16* kcache, ts_bf16* vcache,
                int T, int nq, int nkv, int d, int Lcap, float base, hipStream_t s);
int launch_copy16(const void* src, void* dst, size_t bytes, hipStream_t s, void* dst2 = nullptr, int host_repeat = 1);
// up to four tensors packed by one launch into the device slot dst and the host-mapped slot dst2
struct CopySegments {
  const void* src[4];
  size_t dst_off16[4];   // offset inside both slots, in 16-byte units
  size_t n16[4];         // length in 16-byte units
  int n;
};
int launch_copy16_multi(const CopySegments& segs, void* dst, void* dst2, hipStream_t s, int host_repeat = 1);
int launch_copy_rows(const void* src, size_t src_stride_bytes, size_t row_bytes, int rows, void* dst, void* dst2,
                     hipStream_t s);

size_t gemm_workspace_bytes(int M, int N, int K);
int launch_gemm(const ts_bf16* A, const ts_bf16* W, const ts_bf16* residual, void* C, bool f32out, int M, int N,
                int K, void* ws, size_t ws_bytes, hipStream_t s);
bool gemm_mfma256_supported(int M, int N, int K);
// gate/up projection with SwiGLU in the epilogue (W = F gate rows then F up rows): writes gate_up [M, 2F] and
// act [M, F] = silu(gate) * up computed from the rounded gate_up values
bool gemm_mfma256_glu_supported(int M, int F, int K);
int launch_gemm_mfma256_glu(const ts_bf16* A, const ts_bf16* W, ts_bf16* gate_up, ts_bf16* act, int M, int F, int K,
                            hipStream_t s);
int launch_gemm_mfma256(const ts_bf16* A, const ts_bf16* W, const ts_bf16* residual, ts_bf16* C, int M, int N, int K,
                        hipStream_t s);
int launch_moe_gemm(const ts_bf16* A, const int32_t* row_map, int row_div, const ts_bf16* W,
                    const int32_t* offsets, ts_bf16* C, int rows, int E, int N, int K, hipStream_t s);

size_t attention_decode_workspace_bytes(int B, int nq, int nkv, int d, int Lcap);
// `counters` (optional): B * nkv zeroed int32 words; with them the chunk merge runs inside the
// same launch (last chunk of a (sequence, kv head) to arrive), and the words are left zeroed.
int launch_attention_decode(const ts_bf16* q, int q_stride, const ts_bf16* kc, const ts_bf16* vc, const int32_t* seq_lens,
                            ts_bf16* out, int B, int nq, int nkv, int d, int Lcap, float scale, void* ws,
                            size_t ws_bytes, hipStream_t s, int32_t* counters = nullptr);
int launch_attention_prefill(const ts_bf16* q, const ts_bf16* k, const ts_bf16* v, int q_stride, int kv_stride,
                             const int32_t* cu, ts_bf16* out, int S, int T, int max_seqlen, int nq, int nkv, int d,
                             float scale, int causal, hipStream_t s);

// router projection for up to 16 experts (one wave per token); larger routers go through launch_gemm
bool moe_router_supported(int E, int H);
int launch_moe_router(const ts_bf16* h, const ts_bf16* w_router, float* logits, int T, int E, int H, hipStream_t s);
int launch_moe_route(const float* logits, int T, int E, int k, int32_t* idx, float* w, int32_t* counts,
                     int32_t* offsets, int32_t* perm, hipStream_t s);
int launch_moe_combine(const ts_bf16* y, const int32_t* perm, const float* w, const ts_bf16* residual, ts_bf16* out,
                       int32_t* inv, int T, int k, int H, hipStream_t s);

}  // namespace ts
