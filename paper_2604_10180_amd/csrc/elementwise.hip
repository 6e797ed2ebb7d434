// Memory-bound row/element kernels: RMSNorm, SwiGLU, RoPE + KV append, boundary pack copy.
// All of them move 16 bytes per lane per access and keep arithmetic in fp32
// (they sit on the bandwidth side of the regime split of Sec. 2.3).
#include "common.hpp"

namespace ts {

// ---------------------------------------------------------------- RMSNorm
// One workgroup per row; the row stays in registers between the reduction and the scaling.
template <int VPT>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const uint4* x, const uint4* __restrict__ gamma,
                                                      uint4* y, int H8, float eps, float inv_h,
                                                      int32_t* __restrict__ zero, int nzero) {
  const int row = blockIdx.x;
  const int tid = threadIdx.x;
  if (row == 0)
    for (int i = tid; i < nzero; i += 256) zero[i] = 0;
  const uint4* xr = x + (size_t)row * H8;
  U4 v[VPT], gm[VPT];
  // the gains do not depend on the reduction: their loads travel together with the row's
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    int c = tid + i * 256;
    if (c < H8) gm[i].u = gamma[c];
  }
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    int c = tid + i * 256;
    if (c < H8) {
      v[i].u = xr[c];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float a = bf_lo(v[i].w[j]), b = bf_hi(v[i].w[j]);
        ss += a * a + b * b;
      }
    }
  }
  __shared__ float red[4];
  ss = wave_sum(ss);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  float tot = red[0] + red[1] + red[2] + red[3];
  float rs = 1.0f / sqrtf(tot * inv_h + eps);
  uint4* yr = y + (size_t)row * H8;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    int c = tid + i * 256;
    if (c < H8) {
      U4 g, o;
      g.u = gm[i].u;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float a = bf_lo(v[i].w[j]) * rs * bf_lo(g.w[j]);
        float b = bf_hi(v[i].w[j]) * rs * bf_hi(g.w[j]);
        o.w[j] = pack_bf16(a, b);
      }
      yr[c] = o.u;
    }
  }
}

int launch_rmsnorm(const ts_bf16* x, const ts_bf16* gamma, ts_bf16* y, int T, int H, float eps, hipStream_t s,
                   int32_t* zero, int nzero) {
  if (T == 0) return TS_OK;
  const int H8 = H / 8;
  const int vpt = cdiv(H8, 256);
  dim3 grid(T), block(256);
  const uint4* xp = reinterpret_cast<const uint4*>(x);
  const uint4* gp = reinterpret_cast<const uint4*>(gamma);
  uint4* yp = reinterpret_cast<uint4*>(y);
  const float inv_h = 1.0f / (float)H;
  if (vpt <= 1) TS_LAUNCH_LAST("rmsnorm", rmsnorm_kernel<1>, grid, block, 0, s, xp, gp, yp, H8, eps, inv_h, zero, nzero);
  else if (vpt <= 2) TS_LAUNCH_LAST("rmsnorm", rmsnorm_kernel<2>, grid, block, 0, s, xp, gp, yp, H8, eps, inv_h, zero, nzero);
  else if (vpt <= 4) TS_LAUNCH_LAST("rmsnorm", rmsnorm_kernel<4>, grid, block, 0, s, xp, gp, yp, H8, eps, inv_h, zero, nzero);
  else if (vpt <= 8) TS_LAUNCH_LAST("rmsnorm", rmsnorm_kernel<8>, grid, block, 0, s, xp, gp, yp, H8, eps, inv_h, zero, nzero);
  else TS_LAUNCH_LAST("rmsnorm", rmsnorm_kernel<16>, grid, block, 0, s, xp, gp, yp, H8, eps, inv_h, zero, nzero);
  TS_LAUNCH_CHECK("rmsnorm");
  return TS_OK;
}

// ---------------------------------------------------------------- SwiGLU
__global__ __launch_bounds__(256) void swiglu_kernel(const uint4* __restrict__ gu, uint4* __restrict__ out,
                                                     long total, int F8) {
  long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  long t = i / F8;
  int c = (int)(i - t * F8);
  const uint4* row = gu + t * (2L * F8);
  U4 g, u, o;
  g.u = row[c];
  u.u = row[F8 + c];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float g0 = bf_lo(g.w[j]), g1 = bf_hi(g.w[j]);
    float a = g0 / (1.0f + __expf(-g0)) * bf_lo(u.w[j]);
    float b = g1 / (1.0f + __expf(-g1)) * bf_hi(u.w[j]);
    o.w[j] = pack_bf16(a, b);
  }
  out[i] = o.u;
}

int launch_swiglu(const ts_bf16* gu, ts_bf16* out, int T, int F, hipStream_t s) {
  if (T == 0) return TS_OK;
  const int F8 = F / 8;
  long total = (long)T * F8;
  dim3 grid((unsigned)((total + 255) / 256)), block(256);
  TS_LAUNCH_LAST("swiglu", swiglu_kernel, grid, block, 0, s, reinterpret_cast<const uint4*>(gu),
                     reinterpret_cast<uint4*>(out), total, F8);
  TS_LAUNCH_CHECK("swiglu");
  return TS_OK;
}

// ---------------------------------------------------------------- RoPE + KV append
// Work item = (token, head, 8 consecutive pair indices): loads the lower-half and
// upper-half 16-byte chunks of the head vector, rotates, stores; k items also write the
// rotated row into the cache; v items copy their chunk into the cache.
__global__ __launch_bounds__(256) void rope_kernel(ts_bf16* __restrict__ q, ts_bf16* __restrict__ k,
                                                   const ts_bf16* __restrict__ v, int q_stride, int kv_stride,
                                                   const int32_t* __restrict__ pos, const int32_t* __restrict__ seq_id,
                                                   const float* __restrict__ cos_sin, int table_len,
                                                   ts_bf16* __restrict__ kcache, ts_bf16* __restrict__ vcache, int nq,
                                                   int nkv, int d, int Lcap, float base) {
  const int t = blockIdx.y;
  const int half8 = d / 16;            // 16-byte chunks per half head
  const int wq = nq * half8, wk = nkv * half8, wv = (vcache != nullptr) ? nkv * (d / 8) : 0;
  const int item = blockIdx.x * 256 + threadIdx.x;
  if (item >= wq + wk + wv) return;
  const int p = pos[t];
  const bool cache_ok = (kcache != nullptr) && p >= 0 && p < Lcap;
  const long sid = (kcache != nullptr) ? (long)seq_id[t] : 0;
  if (item >= wq + wk) {  // v chunk copy
    int it = item - wq - wk;
    int h = it / (d / 8), c = it % (d / 8);
    if (cache_ok) {
      uint4 val = ldg16(v + (size_t)t * kv_stride + h * d + c * 8);
      stg16(vcache + ((sid * nkv + h) * (long)Lcap + p) * d + c * 8, val);
    }
    return;
  }
  const bool is_k = item >= wq;
  const int it = is_k ? item - wq : item;
  const int h = it / half8, c = it % half8;
  ts_bf16* vec = (is_k ? k + (size_t)t * kv_stride : q + (size_t)t * q_stride) + h * d;
  U4 lo, hi, olo, ohi;
  lo.u = ldg16(vec + c * 8);
  hi.u = ldg16(vec + d / 2 + c * 8);
  float cs[8], sn[8];
  if (cos_sin != nullptr && p >= 0 && p < table_len) {
    const float4* row = reinterpret_cast<const float4*>(cos_sin + (size_t)p * d);
    float4 c0 = row[c * 2], c1 = row[c * 2 + 1];
    float4 s0 = row[d / 8 + c * 2], s1 = row[d / 8 + c * 2 + 1];
    cs[0] = c0.x; cs[1] = c0.y; cs[2] = c0.z; cs[3] = c0.w; cs[4] = c1.x; cs[5] = c1.y; cs[6] = c1.z; cs[7] = c1.w;
    sn[0] = s0.x; sn[1] = s0.y; sn[2] = s0.z; sn[3] = s0.w; sn[4] = s1.x; sn[5] = s1.y; sn[6] = s1.z; sn[7] = s1.w;
  } else {
    const double lb = log2((double)base);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int i = c * 8 + j;
      double theta = exp2(-2.0 * (double)i / (double)d * lb);
      double ang = (double)p * theta;
      cs[j] = (float)cos(ang);
      sn[j] = (float)sin(ang);
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float a0 = bf_lo(lo.w[j]), a1 = bf_hi(lo.w[j]);
    float b0 = bf_lo(hi.w[j]), b1 = bf_hi(hi.w[j]);
    olo.w[j] = pack_bf16(a0 * cs[2 * j] - b0 * sn[2 * j], a1 * cs[2 * j + 1] - b1 * sn[2 * j + 1]);
    ohi.w[j] = pack_bf16(b0 * cs[2 * j] + a0 * sn[2 * j], b1 * cs[2 * j + 1] + a1 * sn[2 * j + 1]);
  }
  stg16(vec + c * 8, olo.u);
  stg16(vec + d / 2 + c * 8, ohi.u);
  if (is_k && cache_ok) {
    ts_bf16* dst = kcache + ((sid * nkv + h) * (long)Lcap + p) * d;
    stg16(dst + c * 8, olo.u);
    stg16(dst + d / 2 + c * 8, ohi.u);
  }
}

int launch_rope(ts_bf16* q, ts_bf16* k, const ts_bf16* v, int q_stride, int kv_stride, const int32_t* pos,
                const int32_t* seq_id, const float* cos_sin, int table_len, ts_bf16* kcache, ts_bf16* vcache, int T,
                int nq, int nkv, int d, int Lcap, float base, hipStream_t s) {
  if (T == 0) return TS_OK;
  const int items = (nq + nkv) * (d / 16) + (vcache ? nkv * (d / 8) : 0);
  dim3 grid(cdiv(items, 256), T), block(256);
  TS_LAUNCH_LAST("rope", rope_kernel, grid, block, 0, s, q, k, v, q_stride, kv_stride, pos, seq_id, cos_sin, table_len,
                     kcache, vcache, nq, nkv, d, Lcap, base);
  TS_LAUNCH_CHECK("rope");
  return TS_OK;
}

// ---------------------------------------------------------------- boundary pack (contiguous copy)
// Reads the boundary tensor once and writes it to the packed device slot and, when given, to the
// device-mapped pinned host slot as well: the transfer is initiated by the kernel itself (the
// analogue of the GPU-initiated sends of Sec. 4), with no copy-engine command whose cross-stream
// dependency the runtime would resolve by blocking the launching host thread.
// host_repeat > 1 writes the whole tensor that many times to the host slot, pass after pass (stores to one
// address back to back would be merged on the way): the bytes over the link are multiplied, i.e. the link looks
// that many times slower (Sec. 5, sensitivity to the interconnect bandwidth).
__global__ __launch_bounds__(256) void copy16_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                     uint4* __restrict__ dst2, size_t n16, int host_repeat) {
  const size_t i0 = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  if (dst2 == nullptr) {
    for (size_t i = i0; i < n16; i += stride) dst[i] = src[i];
    return;
  }
  for (size_t i = i0; i < n16; i += stride) {
    const uint4 v = src[i];
    dst[i] = v;
    dst2[i] = v;
  }
  for (int r = 1; r < host_repeat; ++r) {
    asm volatile("" ::: "memory");
    for (size_t i = i0; i < n16; i += stride) dst2[i] = src[i];
  }
}

// Several boundary tensors in one launch (segments are consecutive in both destination slots).
__global__ __launch_bounds__(256) void copy16_multi_kernel(CopySegments segs, uint4* __restrict__ dst,
                                                           uint4* __restrict__ dst2, int host_repeat) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (int r = 0; r < host_repeat; ++r) {
    for (int g = 0; g < segs.n; ++g) {
      const uint4* src = reinterpret_cast<const uint4*>(segs.src[g]);
      const size_t base = segs.dst_off16[g], n16 = segs.n16[g];
      for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const uint4 v = src[i];
        if (r == 0) dst[base + i] = v;
        dst2[base + i] = v;
      }
    }
    asm volatile("" ::: "memory");
  }
}

int launch_copy16_multi(const CopySegments& segs, void* dst, void* dst2, hipStream_t s, int host_repeat) {
  if (segs.n == 0) return TS_OK;
  // Four workgroups: the bandwidth-bound compute kernels beside it run one or two workgroups per CU and end
  // when their slowest CU ends, so every CU the pack kernel's PCIe stores sit on costs them time (measured on
  // the 70B pipelined step: 2 or 4 workgroups +4.5 % over the copy-free step, 32: +6.5 %, 512 single-wave
  // ones: +8.5 %; one workgroup cannot keep up with the step).
  TS_LAUNCH("copy16", copy16_multi_kernel, dim3(4), dim3(256), 0, s, segs, reinterpret_cast<uint4*>(dst),
            reinterpret_cast<uint4*>(dst2), host_repeat);
  TS_LAUNCH_CHECK("copy16");
  return TS_OK;
}

// `rows` rows of row16 16-byte units each, src_stride16 units apart, packed densely into dst and dst2.
__global__ __launch_bounds__(256) void copy_rows_kernel(const uint4* __restrict__ src, size_t src_stride16, size_t row16,
                                                        size_t rows, uint4* __restrict__ dst, uint4* __restrict__ dst2) {
  const size_t total = rows * row16, stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
    const size_t r = i / row16, c = i - r * row16;
    const uint4 v = src[r * src_stride16 + c];
    dst[i] = v;
    dst2[i] = v;
  }
}

int launch_copy_rows(const void* src, size_t src_stride_bytes, size_t row_bytes, int rows, void* dst, void* dst2,
                     hipStream_t s) {
  if (rows == 0 || row_bytes == 0) return TS_OK;
  TS_REQUIRE(src_stride_bytes % 16 == 0 && row_bytes % 16 == 0 && aligned16(src), TS_ERR_INVALID_ARG,
             "copy_rows: rows must be whole 16-byte units");
  const size_t total = (size_t)rows * (row_bytes / 16);
  unsigned blocks = (unsigned)((total + 255) / 256);
  if (blocks > 8) blocks = 8;   // background traffic: a few workgroups, it must not take CUs from the compute streams
  TS_LAUNCH("copy_rows", copy_rows_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<const uint4*>(src),
            src_stride_bytes / 16, row_bytes / 16, (size_t)rows, reinterpret_cast<uint4*>(dst), reinterpret_cast<uint4*>(dst2));
  TS_LAUNCH_CHECK("copy_rows");
  return TS_OK;
}

int launch_copy16(const void* src, void* dst, size_t bytes, hipStream_t s, void* dst2, int host_repeat) {
  if (bytes == 0) return TS_OK;
  size_t n16 = bytes / 16;
  unsigned blocks = (unsigned)((n16 + 255) / 256);
  // few workgroups when the copy leaves over PCIe: it must not take CUs from the compute streams
  const unsigned cap = dst2 != nullptr ? 4 : 2048;
  if (blocks > cap) blocks = cap;
  TS_LAUNCH("copy16", copy16_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<const uint4*>(src),
            reinterpret_cast<uint4*>(dst), reinterpret_cast<uint4*>(dst2), n16, host_repeat);
  TS_LAUNCH_CHECK("copy16");
  return TS_OK;
}

}  // namespace ts
