// Causal prefill attention over packed fresh sequences (the compute-bound tiled kernel of
// Sec. 2.3), flash-style: keys are visited in blocks of 64 with an online softmax, nothing of
// size L x L is materialised.
//
// Workgroup = 4 waves (one per SIMD) = one kv head x the query heads that share it x
// consecutive 32-query blocks; two workgroups fit a CU, so each SIMD holds two waves of
// unrelated workgroups that drift apart and fill each other's softmax and barrier gaps (an
// 8-wave workgroup with a three-stage ring, still selectable through the NW template
// parameter, measured the same speed).  With the usual group of 4 query heads a workgroup is
// 4 heads x 32 queries, so all its waves stop at the same causal boundary.
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
static_assert(3 * kImgU4PerWave <= kStageU4, "three per-wave output images must fit one ring stage");

// Separate LDS variables per ring stage: direct loads into one provably do not alias operand
// reads from the other, so those reads are not made to wait for the loads in flight.
__shared__ uint4 g_kv0[kStageU4];
__shared__ uint4 g_kv1[kStageU4];
__shared__ uint4 g_kv2[kStageU4];

// s_waitcnt on the vector-memory counter only (N <= 15): at most N loads of this wave still in flight
template <int N> __device__ __forceinline__ void wait_vm() { __builtin_amdgcn_s_waitcnt(0x0F70 | N); }

// chunk swizzles (row = key index inside the block)
template <int D> __device__ __forceinline__ int kswz(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
template <int D> __device__ __forceinline__ int vswz(int row) { return D == 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1); }

template <int D, int NW>
__device__ __forceinline__ void attn_prefill_body(const ts_bf16* __restrict__ q, const ts_bf16* __restrict__ k,
                                                  const ts_bf16* __restrict__ v, int q_stride, int kv_stride,
                                                  const int32_t* __restrict__ cu, ts_bf16* __restrict__ out, int nq,
                                                  int nkv, int hpw, int nseq, int nqb, float c_scale,
                                                  int causal) {
  constexpr int KB = kKeysPerBlock;
  constexpr int STEPS = D / 16;        // 16-wide d steps of the QK product
  constexpr int DT = D / 32;           // 32-wide output column tiles
  constexpr int CPR = D / 8;           // 16-byte chunks per row
  constexpr int ROWB = D * 2;          // bytes per row
  constexpr int RPI = 1024 / ROWB;     // rows per direct-load instruction
  constexpr int LPW = KB / RPI / NW;   // direct loads per wave per tile
  constexpr int VT = KB * ROWB;        // byte offset of the V tile inside a stage
  constexpr int IMGROW = ROWB + kImgRowPad;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r32 = lane & 31, g = lane >> 5;
  const int group = nq / nkv;
  const int qsubs = NW / hpw;                      // 32-query blocks per workgroup
  const int QB = 32 * qsubs;
  const int head_local = wave % hpw, qsub = wave / hpw;
  const int hgroups = group / hpw;
  // Workgroup id -> (head group, sequence) fastest, query block slowest and descending: the long
  // (late) query blocks are scheduled first, and because consecutive ids go round-robin to the
  // 8 XCDs every XCD gets the same mix of block lengths while one (kv head, sequence) keeps
  // landing on the same XCD, whose L2 then serves its K/V to all query blocks.
  const int npairs = nkv * hgroups * nseq;
  const int pair = blockIdx.x % npairs;
  const int qb = nqb - 1 - blockIdx.x / npairs;
  const int sq = pair / (nkv * hgroups), hy = pair % (nkv * hgroups);
  const int kvh = hy / hgroups, hg = hy % hgroups;
  const int h = kvh * group + hg * hpw + head_local;
  const int a = cu[sq], n = cu[sq + 1] - a;
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
  uint32_t ld_koff[LPW], ld_voff[LPW];      // byte offsets from the first key of a block (full blocks)
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int row = (i * NW + wave) * RPI + lane / CPR, p = lane % CPR;
    ld_row[i] = row;
    ld_kc[i] = (p ^ kswz<D>(row)) * 8;
    ld_vc[i] = (p ^ vswz<D>(row)) * 8;
    ld_koff[i] = ((uint32_t)row * (uint32_t)kv_stride + ld_kc[i]) * 2u;
    ld_voff[i] = ((uint32_t)row * (uint32_t)kv_stride + ld_vc[i]) * 2u;
  }
  auto issue = [&](uint4* stage, int kb) {
    if (kb * KB + KB <= n) {   // full block: uniform base + per-lane constant offset, no address arithmetic
      const char* kb_base = reinterpret_cast<const char*>(kbase) + (size_t)kb * KB * kv_stride * 2;
      const char* vb_base = reinterpret_cast<const char*>(vbase) + (size_t)kb * KB * kv_stride * 2;
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        uint4* dst = stage + (i * NW + wave) * 64;
        __builtin_amdgcn_global_load_lds(kb_base + ld_koff[i], (lds_void*)dst, 16, 0, 0);
        __builtin_amdgcn_global_load_lds(vb_base + ld_voff[i], (lds_void*)(dst + VT / 16), 16, 0, 0);
      }
    } else {                   // last, partial block: rows past the end re-read the last key (masked later)
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        const size_t key = (size_t)min(kb * KB + ld_row[i], n - 1);
        uint4* dst = stage + (i * NW + wave) * 64;
        __builtin_amdgcn_global_load_lds(kbase + key * kv_stride + ld_kc[i], (lds_void*)dst, 16, 0, 0);
        __builtin_amdgcn_global_load_lds(vbase + key * kv_stride + ld_vc[i], (lds_void*)(dst + VT / 16), 16, 0, 0);
      }
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
    // K fragments run three d-steps ahead of the MFMAs that consume them
    U4 kf[STEPS][2];
    auto load_k = [&](int sp) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
        kf[sp][t].u = *reinterpret_cast<const uint4*>(st + t * 32 * ROWB + krow + (((sp * 2 + g) ^ kx) * 16));
    };
    load_k(0);
    load_k(1);
    load_k(2);
#pragma unroll
    for (int sp = 0; sp < STEPS; ++sp) {
      __builtin_amdgcn_sched_barrier(0);
      if (sp + 3 < STEPS) load_k(sp + 3);
#pragma unroll
      for (int t = 0; t < 2; ++t) s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[sp][t].b, qf[sp].b, s[t], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
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
    // ---- online softmax.  Scores stay raw; c_scale = scale * log2(e) enters the exponent.
    // The reference maximum m_run is moved only when some score of the block would exceed it by
    // more than 8 binades (p <= 256 keeps bf16's relative precision and is far from fp32
    // overflow in the row sum); o / l does not depend on which reference is used, and the 64
    // accumulator rescales are then skipped for almost every block.
    float bm = s[0][0];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) bm = fmaxf(bm, s[t][e]);
    bm = fmaxf(bm, __shfl_xor(bm, 32, 64));            // finite from the first block on (key 0 is visible)
    if (__builtin_amdgcn_ballot_w64((bm - m_run) * c_scale > 8.0f) != 0) {
      const float m_new = fmaxf(m_run, bm);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c_scale);   // first block: exp2(-inf) = 0
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
      m_run = m_new;
    }
    const float mc = m_run * c_scale;
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
  // One ring step.  Eight waves use three stages: prefetch block kb+2 into the stage that was
  // read in step kb-1 (past the end the final block is fetched again into an idle stage rather
  // than branching), compute block kb, then wait until block kb+1 has landed: only the loads
  // issued in this step may still be in flight.  Four waves (two workgroups per CU, half the
  // LDS each) use two stages and wait for everything.
  constexpr int AHEAD = (NW == 8) ? 2 : 1;
  auto step = [&](const uint4* cur, uint4* tgt, int kb) {
    issue(tgt, min(kb + AHEAD, nkb - 1));
    __builtin_amdgcn_sched_barrier(0);
    if (!(causal && kb * KB > q0 + 31)) block(cur, kb);   // keys entirely above this wave's diagonal: skip
    wait_vm<(AHEAD - 1) * 2 * LPW>();
    __syncthreads();
  };

  int kb = 0;
  if constexpr (NW == 8) {
    issue(g_kv0, 0);
    issue(g_kv1, min(1, nkb - 1));
    wait_vm<2 * LPW>();
    __syncthreads();
    for (; kb + 3 <= nkb; kb += 3) {
      step(g_kv0, g_kv2, kb);
      step(g_kv1, g_kv0, kb + 1);
      step(g_kv2, g_kv1, kb + 2);
    }
    if (kb < nkb) {
      step(g_kv0, g_kv2, kb);
      if (kb + 1 < nkb) step(g_kv1, g_kv0, kb + 1);
    }
  } else {
    issue(g_kv0, 0);
    wait_vm<0>();
    __syncthreads();
    for (; kb + 2 <= nkb; kb += 2) {
      step(g_kv0, g_kv1, kb);
      step(g_kv1, g_kv0, kb + 1);
    }
    if (kb < nkb) step(g_kv0, g_kv1, kb);
  }
  wait_vm<0>();        // the trailing re-fetches have landed,
  __syncthreads();     // and every wave is done with the ring: it now holds the output images

  // ---- epilogue: normalise, round, transpose through this wave's LDS image, store whole rows
  l_run += __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_run;
  uint4* img_stage = wave < 3 ? g_kv0 : g_kv1;
  if constexpr (NW == 8) img_stage = wave < 3 ? g_kv0 : (wave < 6 ? g_kv1 : g_kv2);
  char* img = reinterpret_cast<char*>(img_stage + (wave % 3) * kImgU4PerWave);
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
#define TS_PREFILL_ARGS const ts_bf16* q, const ts_bf16* k, const ts_bf16* v, int q_stride, int kv_stride, \
                        const int32_t* cu, ts_bf16* out, int nq, int nkv, int hpw, int nseq, int nqb, float c_scale, int causal
#define TS_PREFILL_PASS q, k, v, q_stride, kv_stride, cu, out, nq, nkv, hpw, nseq, nqb, c_scale, causal
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_prefill_d128_w4_kernel(TS_PREFILL_ARGS) {
  attn_prefill_body<128, 4>(TS_PREFILL_PASS);
}
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_prefill_d64_w4_kernel(TS_PREFILL_ARGS) {
  attn_prefill_body<64, 4>(TS_PREFILL_PASS);
}


int launch_attention_prefill(const ts_bf16* q, const ts_bf16* k, const ts_bf16* v, int q_stride, int kv_stride,
                             const int32_t* cu, ts_bf16* out, int S, int T, int max_seqlen, int nq, int nkv, int d,
                             float scale, int causal, hipStream_t s) {
  if (S == 0 || T == 0 || max_seqlen == 0) return TS_OK;
  const float c_scale = scale * 1.4426950408889634f;
  // query heads per workgroup: the largest power of two (<= waves) that divides the GQA group
  constexpr int NW = 4;
  const int group = nq / nkv;
  int hpw = 1;
  while (hpw < NW && group % (hpw * 2) == 0) hpw *= 2;
  const int QB = 32 * (NW / hpw);
  const int nqb = cdiv(max_seqlen, QB);
  dim3 grid(nqb * nkv * (group / hpw) * S);
#define TS_PREFILL_LAUNCH(kern, threads) \
  TS_LAUNCH_LAST("attn_prefill", kern, grid, dim3(threads), 0, s, q, k, v, q_stride, kv_stride, cu, out, nq, nkv, hpw, S, nqb, c_scale, causal)
  if (d == 128) TS_PREFILL_LAUNCH(attn_prefill_d128_w4_kernel, 256);
  else TS_PREFILL_LAUNCH(attn_prefill_d64_w4_kernel, 256);
  TS_LAUNCH_CHECK("attn_prefill");
  return TS_OK;
}

}  // namespace ts
