// MoE routing (exact integer outputs, deterministic grouping) and weighted combine.
#include "common.hpp"

namespace ts {

// Router logits for a handful of experts (E <= 16): logits[t, e] = h[t, :] . Wr[e, :] in fp32.  One workgroup
// per token; a thread takes every 256th 16-byte chunk of the row against the same chunk of all E router rows
// (64 KB at E = 8, H = 4096: served by the caches); the E sums are reduced across the wave, then across the
// four waves through LDS in wave order.  As a GEMM this is a single 8-column tile, i.e. eight workgroups
// after splitting K.
template <int EMAX>
__global__ __launch_bounds__(256) void moe_router_kernel(const uint4* __restrict__ h, const uint4* __restrict__ wr,
                                                         float* __restrict__ logits, int T, int E, int H8) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = blockIdx.x;
  float acc[EMAX];
#pragma unroll
  for (int e = 0; e < EMAX; ++e) acc[e] = 0.f;
  const uint4* row = h + (size_t)t * H8;
  for (int c = tid; c < H8; c += 256) {
    U4 x;
    x.u = row[c];
    float xf[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) { xf[2 * j] = bf_lo(x.w[j]); xf[2 * j + 1] = bf_hi(x.w[j]); }
    // rows past E re-read the last router row (their sums are never stored): no branch, so all loads of a chunk
    // are in flight together
    U4 w[EMAX];
#pragma unroll
    for (int e = 0; e < EMAX; ++e) w[e].u = wr[(size_t)(e < E ? e : E - 1) * H8 + c];
#pragma unroll
    for (int e = 0; e < EMAX; ++e)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[e] += xf[2 * j] * bf_lo(w[e].w[j]) + xf[2 * j + 1] * bf_hi(w[e].w[j]);
  }
  __shared__ float part[4][EMAX];
#pragma unroll
  for (int e = 0; e < EMAX; ++e) {
    const float v = wave_sum(acc[e]);
    if (lane == 0) part[wave][e] = v;
  }
  __syncthreads();
  if (tid < E) logits[(size_t)t * E + tid] = ((part[0][tid] + part[1][tid]) + part[2][tid]) + part[3][tid];
}

bool moe_router_supported(int E, int H) { return E >= 1 && E <= 16 && H % 8 == 0; }

int launch_moe_router(const ts_bf16* h, const ts_bf16* w_router, float* logits, int T, int E, int H, hipStream_t s) {
  if (T == 0) return TS_OK;
  const uint4* hp = reinterpret_cast<const uint4*>(h);
  const uint4* wp = reinterpret_cast<const uint4*>(w_router);
  if (E <= 8) TS_LAUNCH("moe_router", moe_router_kernel<8>, dim3(T), dim3(256), 0, s, hp, wp, logits, T, E, H / 8);
  else TS_LAUNCH("moe_router", moe_router_kernel<16>, dim3(T), dim3(256), 0, s, hp, wp, logits, T, E, H / 8);
  TS_LAUNCH_CHECK("moe_router");
  return TS_OK;
}

// One thread per token: k rounds of "largest remaining logit, lowest index on ties".
__global__ __launch_bounds__(256) void moe_topk_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                       int32_t* __restrict__ idx, float* __restrict__ w) {
  int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const float* l = logits + (size_t)t * E;
  unsigned long long taken = 0ull;
  float first = 0.f, sum = 0.f;
  float sel[64];
  for (int s = 0; s < k; ++s) {
    int best = -1;
    float bv = 0.f;
    for (int e = 0; e < E; ++e) {
      if ((taken >> e) & 1ull) continue;
      float v = l[e];
      if (best < 0 || v > bv) { best = e; bv = v; }
    }
    taken |= 1ull << best;
    idx[(size_t)t * k + s] = best;
    if (s == 0) first = bv;
    float ex = expf(bv - first);
    sel[s] = ex;
    sum += ex;
  }
  for (int s = 0; s < k; ++s) w[(size_t)t * k + s] = sel[s] / sum;
}

// One workgroup per expert e: counts assignments below e and equal to e, then lists the
// assignments of e in ascending order (stable), so perm is deterministic.
__global__ __launch_bounds__(256) void moe_group_kernel(const int32_t* __restrict__ idx, int n, int E,
                                                        int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                        int32_t* __restrict__ perm) {
  const int e = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  __shared__ int s_lt[4], s_eq[4], s_base, s_wave[4];
  int lt = 0, eq = 0;
  for (int a = tid; a < n; a += 256) {
    int v = idx[a];
    lt += (v < e);
    eq += (v == e);
  }
  for (int o = 32; o > 0; o >>= 1) {
    lt += __shfl_xor(lt, o, 64);
    eq += __shfl_xor(eq, o, 64);
  }
  if (lane == 0) { s_lt[wv] = lt; s_eq[wv] = eq; }
  __syncthreads();
  const int base = s_lt[0] + s_lt[1] + s_lt[2] + s_lt[3];
  const int cnt = s_eq[0] + s_eq[1] + s_eq[2] + s_eq[3];
  if (tid == 0) {
    counts[e] = cnt;
    offsets[e] = base;
    if (e == E - 1) offsets[E] = base + cnt;
    s_base = 0;
  }
  __syncthreads();
  for (int a0 = 0; a0 < n; a0 += 256) {
    int a = a0 + tid;
    bool flag = (a < n) && (idx[a] == e);
    unsigned long long m = __ballot(flag);
    int before = __popcll(m & ((1ull << lane) - 1ull));
    if (lane == 0) s_wave[wv] = __popcll(m);
    __syncthreads();
    int wbase = 0;
    for (int i = 0; i < wv; ++i) wbase += s_wave[i];
    int run = s_base;
    if (flag) perm[base + run + wbase + before] = a;
    __syncthreads();
    if (tid == 0) s_base = run + s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
    __syncthreads();
  }
}

int launch_moe_route(const float* logits, int T, int E, int k, int32_t* idx, float* w, int32_t* counts,
                     int32_t* offsets, int32_t* perm, hipStream_t s) {
  if (T > 0) {
    TS_LAUNCH("moe_topk", moe_topk_kernel, dim3(cdiv(T, 256)), dim3(256), 0, s, logits, T, E, k, idx, w);
    TS_LAUNCH_CHECK("moe_topk");
  }
  TS_LAUNCH("moe_group", moe_group_kernel, dim3(E), dim3(256), 0, s, idx, T * k, E, counts, offsets, perm);
  TS_LAUNCH_CHECK("moe_group");
  return TS_OK;
}

// inv[perm[r]] = r
__global__ __launch_bounds__(256) void moe_invert_kernel(const int32_t* __restrict__ perm, int32_t* __restrict__ inv,
                                                         int n) {
  int r = blockIdx.x * 256 + threadIdx.x;
  if (r < n) inv[perm[r]] = r;
}

// out[t] = residual[t] + sum_s w[t,s] * y[inv[t*k+s]], slots added in ascending s (deterministic).
__global__ __launch_bounds__(256) void moe_combine_kernel(const uint4* __restrict__ y, const int32_t* __restrict__ inv,
                                                          const float* __restrict__ w, const uint4* __restrict__ res,
                                                          uint4* __restrict__ out, long total, int H8, int k) {
  long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  long t = i / H8;
  int c = (int)(i - t * H8);
  float acc[8];
  if (res != nullptr) {
    U4 r;
    r.u = res[i];
#pragma unroll
    for (int j = 0; j < 4; ++j) { acc[2 * j] = bf_lo(r.w[j]); acc[2 * j + 1] = bf_hi(r.w[j]); }
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  }
  for (int s = 0; s < k; ++s) {
    int r = inv[t * k + s];
    float ws = w[t * k + s];
    U4 v;
    v.u = y[(long)r * H8 + c];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[2 * j] += ws * bf_lo(v.w[j]);
      acc[2 * j + 1] += ws * bf_hi(v.w[j]);
    }
  }
  U4 o;
#pragma unroll
  for (int j = 0; j < 4; ++j) o.w[j] = pack_bf16(acc[2 * j], acc[2 * j + 1]);
  out[i] = o.u;
}

int launch_moe_combine(const ts_bf16* y, const int32_t* perm, const float* w, const ts_bf16* residual, ts_bf16* out,
                       int32_t* inv, int T, int k, int H, hipStream_t s) {
  if (T == 0) return TS_OK;
  int n = T * k;
  TS_LAUNCH("moe_invert", moe_invert_kernel, dim3(cdiv(n, 256)), dim3(256), 0, s, perm, inv, n);
  TS_LAUNCH_CHECK("moe_invert");
  const int H8 = H / 8;
  long total = (long)T * H8;
  TS_LAUNCH_LAST("moe_combine", moe_combine_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                     reinterpret_cast<const uint4*>(y), inv, w, reinterpret_cast<const uint4*>(residual),
                     reinterpret_cast<uint4*>(out), total, H8, k);
  TS_LAUNCH_CHECK("moe_combine");
  return TS_OK;
}

}  // namespace ts
