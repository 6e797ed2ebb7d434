// Causal prefill attention over packed fresh sequences (the compute-bound tiled kernel of
// Sec. 2.3), flash-style: keys are visited in blocks of 64 with an online softmax, nothing of
// size L x L is materialised.
//
// Workgroup = 8 waves (two per SIMD: one wave's softmax arithmetic overlaps the other's
// MFMAs) = one kv head x the query heads that share it x consecutive 32-query blocks.  With
// the usual group of 4 query heads that is 4 heads x 64 queries, so a staged K/V block is used
// by 256 query rows and all waves of a query block stop at the same causal boundary.
//
// Orientation (32x32x16 bf16 MFMA throughout):
//   S^T[key, query] = K . Q^T      A = K rows from LDS, B = Q fragments held in registers
//   O^T[dcol, query] += V^T . P^T  A = V^T through the LDS transpose read, B = P from registers
// A lane therefore owns ONE query column: its 32 scores of a block, the running max/sum and
// all its output columns sit in its own registers; the only cross-lane step per block is one
// exchange of the block max between the two lane halves.  P needs no data movement between
// the two products: the key -> k-slot assignment of the second product is chosen to be the
// accumulator layout of the first.
//
// K and V blocks (64 keys, row-major) are filled by direct global->LDS loads into a two-stage
// ring; rows are unpadded and bank conflicts are avoided by XOR-swizzling the 16-byte chunks on
// the global side (one pattern for K, read by rows, another for V, read through 4-row
// transposing reads).  The output tile goes through a per-wave LDS image so that it leaves as
// whole 256-byte rows.
#include "common.hpp"

namespace ts {

namespace {

typedef __attribute__((address_space(3))) void lds_void;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kKeysPerBlock = 64;
constexpr int kStageU4 = 2 * kKeysPerBlock * 16;          // K tile + V tile at d = 128: 32 KiB
constexpr int kImgRowPad = 8;                             // bytes of padding per output-image row
constexpr int kImgU4PerWave = 32 * (256 + kImgRowPad) / 16;

// Separate LDS variables per ring stage: direct loads into one provably do not alias operand
// reads from the other, so those reads are not made to wait for the loads in flight.
__shared__ uint4 g_kv0[kStageU4];
__shared__ uint4 g_kv1[kStageU4];
__shared__ uint4 g_oimg[8 * kImgU4PerWave];

__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0) only

// chunk swizzles (row = key index inside the block)
template <int D> __device__ __forceinline__ int kswz(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
template <int D> __device__ __forceinline__ int vswz(int row) { return D == 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1); }

template <int D>
__device__ __forceinline__ void attn_prefill_body(const ts_bf16* __restrict__ q, const ts_bf16* __restrict__ k,
                                                  const ts_bf16* __restrict__ v, int q_stride, int kv_stride,
                                                  const int32_t* __restrict__ cu, ts_bf16* __restrict__ out, int nq,
                                                  int nkv, int hpw, float c_scale, int causal) {
  constexpr int KB = kKeysPerBlock;
  constexpr int STEPS = D / 16;        // 16-wide d steps of the QK product
  constexpr int DT = D / 32;           // 32-wide output column tiles
  constexpr int CPR = D / 8;           // 16-byte chunks per row
  constexpr int ROWB = D * 2;          // bytes per row
  constexpr int RPI = 1024 / ROWB;     // rows per direct-load instruction
  constexpr int LPW = KB / RPI / 8;    // direct loads per wave per tile
  constexpr int VT = KB * ROWB;        // byte offset of the V tile inside a stage
  constexpr int IMGROW = ROWB + kImgRowPad;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r32 = lane & 31, g = lane >> 5;
  const int group = nq / nkv;
  const int qsubs = 8 / hpw;                      // 32-query blocks per workgroup
  const int QB = 32 * qsubs;
  const int head_local = wave % hpw, qsub = wave / hpw;
  const int hgroups = group / hpw;
  const int kvh = blockIdx.y / hgroups, hg = blockIdx.y % hgroups;
  const int h = kvh * group + hg * hpw + head_local;
  const int sq = blockIdx.z;
  const int a = cu[sq], n = cu[sq + 1] - a;
  const int qb = gridDim.x - 1 - blockIdx.x;       // long (late) query blocks are scheduled first
  if (qb * QB >= n) return;
  const int q0 = qb * QB + qsub * 32;             // first query of this wave
  const int qi = q0 + r32;                        // this lane's query
  const int kmax = causal ? min(n, qb * QB + QB) : n;
  const int nkb = (kmax + KB - 1) / KB;

  // ---- Q fragments: B operand, lane (query r32, half g) holds d = s*16 + g*8 .. +8 of step s
  U4 qf[STEPS];
  {
    const ts_bf16* qrow = q + (size_t)(a + min(qi, n - 1)) * q_stride + (size_t)h * D + g * 8;
#pragma unroll
    for (int s = 0; s < STEPS; ++s) qf[s].u = ldg16(qrow + s * 16);
  }

  // ---- direct-load assignment: load i of wave w fills rows (i*8 + w)*RPI .. +RPI of a tile
  const ts_bf16* kbase = k + (size_t)a * kv_stride + (size_t)kvh * D;
  const ts_bf16* vbase = v + (size_t)a * kv_stride + (size_t)kvh * D;
  int ld_row[LPW], ld_kc[LPW], ld_vc[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int row = (i * 8 + wave) * RPI + lane / CPR, p = lane % CPR;
    ld_row[i] = row;
    ld_kc[i] = (p ^ kswz<D>(row)) * 8;
    ld_vc[i] = (p ^ vswz<D>(row)) * 8;
  }
  auto issue = [&](uint4* stage, int kb) {
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      const size_t key = (size_t)min(kb * KB + ld_row[i], n - 1);
      uint4* dst = stage + (i * 8 + wave) * 64;
      __builtin_amdgcn_global_load_lds(kbase + key * kv_stride + ld_kc[i], (lds_void*)dst, 16, 0, 0);
      __builtin_amdgcn_global_load_lds(vbase + key * kv_stride + ld_vc[i], (lds_void*)(dst + VT / 16), 16, 0, 0);
    }
  };

  // ---- operand addresses inside a stage
  // K fragment (tile t, step s): row t*32 + r32, logical chunk s*2 + g
  const int kx = kswz<D>(r32);
  const int krow = r32 * ROWB;
  // V^T fragment through the transposing read: within a 16-lane group, lane j supplies
  // row j/4, columns (j%4)*4 .. +4 and lane i receives column i of those four rows.
  const int j16 = lane & 15;
  const int vrow_l = j16 >> 2;                         // key row inside the 4-row group
  const int dbase = ((lane >> 4) & 1) * 16;            // which 16 output columns of the 32-wide tile
  const int vc = dbase / 8 + ((j16 & 3) >> 1);         // logical chunk inside the tile's 4 chunks
  const int vxq = vswz<D>(vrow_l) / 4;                 // swizzle acts on the tile index
  int voff[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
    voff[dt] = VT + (4 * g + vrow_l) * ROWB + ((dt ^ vxq) * 64 + vc * 16) + (j16 & 1) * 8;

  float m_run = -INFINITY, l_run = 0.f;   // l_run: this lane's own keys only; halves are added at the end
  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;

  auto block = [&](const uint4* stage, int kb) {
    const char* st = reinterpret_cast<const char*>(stage);
    // ---- S^T = K . Q^T : two 32-key tiles
    f32x16 s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) s[t][e] = 0.f;
#pragma unroll
    for (int sp = 0; sp < STEPS; ++sp) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        U4 kf;
        kf.u = *reinterpret_cast<const uint4*>(st + t * 32 * ROWB + krow + (((sp * 2 + g) ^ kx) * 16));
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.b, qf[sp].b, s[t], 0, 0, 0);
      }
    }
    // ---- masking: only blocks that reach the causal diagonal or the end of the sequence
    const int key0 = kb * KB + g * 4;                  // key of (t, e): key0 + t*32 + (e/4)*8 + e%4
    const bool need_mask = (kb * KB + KB > n) || (causal && kb * KB + KB - 1 > q0);
    if (need_mask) {
      const int lim = causal ? min(qi, n - 1) : n - 1;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (key0 + t * 32 + (e >> 2) * 8 + (e & 3) > lim) s[t][e] = -INFINITY;
    }
    // ---- online softmax (scores stay raw; c_scale = scale * log2(e) enters the exponent)
    float bm = s[0][0];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) bm = fmaxf(bm, s[t][e]);
    bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
    const float m_new = fmaxf(m_run, bm);              // finite from the first block on (key 0 is visible)
    const float mc = m_new * c_scale;
    float ps = 0.f;
    U4 pf[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) {
          const float p0 = __builtin_amdgcn_exp2f(s[t][c * 8 + w2 * 2] * c_scale - mc);
          const float p1 = __builtin_amdgcn_exp2f(s[t][c * 8 + w2 * 2 + 1] * c_scale - mc);
          ps += p0 + p1;
          pf[t][c].w[w2] = pack_bf16(p0, p1);
        }
    if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {   // rescale only when some lane's max moved
      const float alpha = __builtin_amdgcn_exp2f(m_run * c_scale - mc);   // first block: exp2(-inf) = 0
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
      m_run = m_new;
    }
    l_run += ps;
    // ---- O^T += V^T . P^T : for product (t, c) the lane's k-slots are the keys of its
    // accumulator elements 8c .. 8c+7 of tile t: rows t*32 + 16c + 4g + {0..3} and + 8
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const char* vp = st + (t * 32 + 16 * c) * ROWB + voff[dt];
          union { bf16x8 b; s16x4 hlf[2]; } vt;
          vt.hlf[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp));
          vt.hlf[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 8 * ROWB));
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt.b, pf[t][c].b, o[dt], 0, 0, 0);
        }
  };
  // one ring step: prefetch the next block (the last step re-fetches the final block into the
  // idle stage rather than branching), compute, then make the prefetched stage visible
  auto step = [&](const uint4* cur, uint4* nxt, int kb) {
    issue(nxt, min(kb + 1, nkb - 1));
    __builtin_amdgcn_sched_barrier(0);
    if (!(causal && kb * KB > q0 + 31)) block(cur, kb);   // keys entirely above this wave's diagonal: skip
    wait_vm0();
    __syncthreads();
  };

  issue(g_kv0, 0);
  wait_vm0();
  __syncthreads();
  int kb = 0;
  for (; kb + 2 <= nkb; kb += 2) {
    step(g_kv0, g_kv1, kb);
    step(g_kv1, g_kv0, kb + 1);
  }
  if (kb < nkb) step(g_kv0, g_kv1, kb);

  // ---- epilogue: normalise, round, transpose through this wave's LDS image, store whole rows
  l_run += __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_run;
  char* img = reinterpret_cast<char*>(g_oimg + wave * kImgU4PerWave);
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      uint2 w;
      w.x = pack_bf16(o[dt][gi * 4 + 0] * inv, o[dt][gi * 4 + 1] * inv);
      w.y = pack_bf16(o[dt][gi * 4 + 2] * inv, o[dt][gi * 4 + 3] * inv);
      *reinterpret_cast<uint2*>(img + r32 * IMGROW + (dt * 32 + gi * 8 + g * 4) * 2) = w;
    }
  // (same wave wrote and reads the image: LDS operations of a wave complete in order)
#pragma unroll
  for (int it = 0; it < 32 / RPI; ++it) {
    const int row = it * RPI + lane / CPR, ch = lane % CPR;
    const uint2 lo = *reinterpret_cast<const uint2*>(img + row * IMGROW + ch * 16);
    const uint2 hi = *reinterpret_cast<const uint2*>(img + row * IMGROW + ch * 16 + 8);
    if (q0 + row < n)
      stg16(out + ((size_t)(a + q0 + row) * nq + h) * D + ch * 8, make_uint4(lo.x, lo.y, hi.x, hi.y));
  }
}

}  // namespace

// (plain kernels around the templated body: the ring stages are namespace-scope LDS variables)
__global__ __launch_bounds__(512) void attn_prefill_d128_kernel(const ts_bf16* q, const ts_bf16* k, const ts_bf16* v,
                                                                int q_stride, int kv_stride, const int32_t* cu,
                                                                ts_bf16* out, int nq, int nkv, int hpw, float c_scale,
                                                                int causal) {
  attn_prefill_body<128>(q, k, v, q_stride, kv_stride, cu, out, nq, nkv, hpw, c_scale, causal);
}
__global__ __launch_bounds__(512) void attn_prefill_d64_kernel(const ts_bf16* q, const ts_bf16* k, const ts_bf16* v,
                                                               int q_stride, int kv_stride, const int32_t* cu,
                                                               ts_bf16* out, int nq, int nkv, int hpw, float c_scale,
                                                               int causal) {
  attn_prefill_body<64>(q, k, v, q_stride, kv_stride, cu, out, nq, nkv, hpw, c_scale, causal);
}

int launch_attention_prefill(const ts_bf16* q, const ts_bf16* k, const ts_bf16* v, int q_stride, int kv_stride,
                             const int32_t* cu, ts_bf16* out, int S, int T, int max_seqlen, int nq, int nkv, int d,
                             float scale, int causal, hipStream_t s) {
  if (S == 0 || T == 0 || max_seqlen == 0) return TS_OK;
  const float c_scale = scale * 1.4426950408889634f;
  // query heads per workgroup: the largest power of two (<= 8) that divides the GQA group
  const int group = nq / nkv;
  int hpw = 1;
  while (hpw < 8 && group % (hpw * 2) == 0) hpw *= 2;
  const int QB = 32 * (8 / hpw);
  dim3 grid(cdiv(max_seqlen, QB), nkv * (group / hpw), S);
  if (d == 128) {
    TS_LAUNCH("attn_prefill", attn_prefill_d128_kernel, grid, dim3(512), 0, s, q, k, v, q_stride, kv_stride, cu, out, nq,
              nkv, hpw, c_scale, causal);
  } else {
    TS_LAUNCH("attn_prefill", attn_prefill_d64_kernel, grid, dim3(512), 0, s, q, k, v, q_stride, kv_stride, cu, out, nq,
              nkv, hpw, c_scale, causal);
  }
  TS_LAUNCH_CHECK("attn_prefill");
  return TS_OK;
}

}  // namespace ts
