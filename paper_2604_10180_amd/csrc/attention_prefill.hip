// Causal prefill attention over packed fresh sequences (the compute-bound tiled kernel of
// Sec. 2.3), flash-style: keys are visited in blocks of 32 with an online softmax, nothing
// of size L x L is materialised.
//
// Same operand orientation as the decode kernel, with 16 queries per wave in place of the
// GQA head group:  S^T[key, query] = K . Q^T  and  O^T[dcol, query] += V^T . P^T, so each lane
// owns one query column for the softmax state.  A workgroup is 4 waves = 64 consecutive
// queries of one (sequence, head); K/V blocks are staged once in LDS for the four waves.
#include "common.hpp"

namespace ts {

template <int D>
__global__ __launch_bounds__(256) void attn_prefill_kernel(const ts_bf16* __restrict__ q, const ts_bf16* __restrict__ k,
                                                           const ts_bf16* __restrict__ v, int q_stride, int kv_stride,
                                                           const int32_t* __restrict__ cu, ts_bf16* __restrict__ out,
                                                           int nq, int nkv, float c_scale, int causal) {
  constexpr int KSTEPS = D / 32, DT = D / 16, CPR = D / 8, ROW = CPR + 1, ROW_H = ROW * 8;
  constexpr int LOADS = 32 * CPR / 256;   // 16-byte chunks per thread per staged block (K and V each)
  const int qb = blockIdx.x, h = blockIdx.y, sq = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, gq = lane >> 4;
  const int a = cu[sq], n = cu[sq + 1] - a;
  if (qb * 64 >= n) return;
  const int kvh = h / (nq / nkv);
  const int kmax = causal ? min(n, qb * 64 + 64) : n;
  const int nkb = (kmax + 31) / 32;

  extern __shared__ uint4 smem[];
  // [2][32][ROW] K then [2][32][ROW] V
  uint4* sK = smem;
  uint4* sV = smem + 2 * 32 * ROW;

  const int qi = qb * 64 + wave * 16 + l16;            // this lane's query column
  U4 qf[KSTEPS];
  {
    const ts_bf16* qrow = q + (size_t)(a + min(qi, n - 1)) * q_stride + (size_t)h * D;
#pragma unroll
    for (int j = 0; j < KSTEPS; ++j) qf[j].u = ldg16(qrow + (j * 4 + gq) * 8);
  }
  const ts_bf16* kbase = k + (size_t)a * kv_stride + (size_t)kvh * D;
  const ts_bf16* vbase = v + (size_t)a * kv_stride + (size_t)kvh * D;

  uint4 kr[LOADS], vr[LOADS];
  auto gload = [&](int kb) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int c = tid + 256 * i;
      const int key = min(kb * 32 + c / CPR, n - 1);
      kr[i] = ldg16(kbase + (size_t)key * kv_stride + (c % CPR) * 8);
      vr[i] = ldg16(vbase + (size_t)key * kv_stride + (c % CPR) * 8);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int c = tid + 256 * i;
      sK[(buf * 32 + c / CPR) * ROW + (c % CPR)] = kr[i];
      sV[(buf * 32 + c / CPR) * ROW + (c % CPR)] = vr[i];
    }
  };

  float m_run = -INFINITY, l_run = 0.f;
  f32x4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  gload(0);
  sstore(0);
  __syncthreads();
  const int wave_qmax = qb * 64 + wave * 16 + 15;
  for (int kb = 0; kb < nkb; ++kb) {
    const int cur = kb & 1;
    if (kb + 1 < nkb) gload(kb + 1);
    const bool active = !(causal && kb * 32 > wave_qmax);
    if (active) {
      f32x4 s[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KSTEPS; ++j) {
          U4 kf;
          kf.u = sK[(cur * 32 + kt * 16 + l16) * ROW + j * 4 + gq];
          s[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.b, qf[j].b, s[kt], 0, 0, 0);
        }
      }
      float sv[8];
      float bm = -INFINITY;
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int key = kb * 32 + (t >> 2) * 16 + gq * 4 + (t & 3);
        const bool ok = (key < n) && (!causal || key <= qi);
        sv[t] = ok ? s[t >> 2][t & 3] * c_scale : -INFINITY;
        bm = fmaxf(bm, sv[t]);
      }
      bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
      bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
      const float m_new = fmaxf(m_run, bm);
      const bool dead = (m_new == -INFINITY);          // no visible key yet for this query column
      const float alpha = dead ? 1.f : exp2f(m_run - m_new);
      float ps = 0.f;
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        sv[t] = dead ? 0.f : exp2f(sv[t] - m_new);
        ps += sv[t];
      }
      l_run = l_run * alpha + ps;
      m_run = m_new;
      U4 pf;
#pragma unroll
      for (int t = 0; t < 4; ++t) pf.w[t] = pack_bf16(sv[2 * t], sv[2 * t + 1]);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
      const uint16_t* vh = reinterpret_cast<const uint16_t*>(sV + (size_t)cur * 32 * ROW);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        U4 vt;
#pragma unroll
        for (int t = 0; t < 8; t += 2) {
          const int key0 = (t >> 2) * 16 + gq * 4 + (t & 3);
          uint32_t lo = vh[key0 * ROW_H + dt * 16 + l16];
          uint32_t hi = vh[(key0 + 1) * ROW_H + dt * 16 + l16];
          vt.w[t >> 1] = lo | (hi << 16);
        }
        o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt.b, pf.b, o[dt], 0, 0, 0);
      }
    }
    if (kb + 1 < nkb) sstore(cur ^ 1);
    __syncthreads();
  }
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (qi < n) {
    const float inv = 1.0f / l_run;
    ts_bf16* orow = out + ((size_t)(a + qi) * nq + h) * D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      uint2 w;
      w.x = pack_bf16(o[dt][0] * inv, o[dt][1] * inv);
      w.y = pack_bf16(o[dt][2] * inv, o[dt][3] * inv);
      *reinterpret_cast<uint2*>(orow + dt * 16 + gq * 4) = w;
    }
  }
}

int launch_attention_prefill(const ts_bf16* q, const ts_bf16* k, const ts_bf16* v, int q_stride, int kv_stride,
                             const int32_t* cu, ts_bf16* out, int S, int T, int max_seqlen, int nq, int nkv, int d,
                             float scale, int causal, hipStream_t s) {
  if (S == 0 || T == 0 || max_seqlen == 0) return TS_OK;
  const float c_scale = scale * 1.4426950408889634f;
  dim3 grid(cdiv(max_seqlen, 64), nq, S);
  if (d == 128) {
    const size_t smem = (size_t)4 * 32 * 17 * sizeof(uint4);
    TS_LAUNCH("attn_prefill", attn_prefill_kernel<128>, grid, dim3(256), smem, s, q, k, v, q_stride, kv_stride, cu, out, nq,
                       nkv, c_scale, causal);
  } else {
    const size_t smem = (size_t)4 * 32 * 9 * sizeof(uint4);
    TS_LAUNCH("attn_prefill", attn_prefill_kernel<64>, grid, dim3(256), smem, s, q, k, v, q_stride, kv_stride, cu, out, nq,
                       nkv, c_scale, causal);
  }
  TS_LAUNCH_CHECK("attn_prefill");
  return TS_OK;
}

}  // namespace ts
