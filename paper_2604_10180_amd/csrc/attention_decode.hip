// Decode attention over the contiguous KV cache: the big bandwidth-bound kernel of a decode
// iteration.  K and V are streamed once from HBM with 16-byte loads; all contractions run on
// the matrix cores so the vector ALU only does the softmax bookkeeping:
//
//   S^T[key, head]  = K[key, :] . Q[head, :]      MFMA 16x16x32, A = K rows via the wave's LDS stage
//   O^T[dcol, head] += V^T[dcol, key] P^T[key, head]  MFMA 16x16x32, A = V^T gathered from LDS
//
// The query heads of one kv head (GQA group, <= 16) fill the N dimension.  With this
// orientation every lane owns one head column for scores, running max, running sum and
// output accumulators, so the online-softmax state needs no cross-lane traffic except a
// 2-step max over the four lane groups.
//
// Split-KV, two forms.  Short caches: grid (chunk, kv head, sequence), a sequence gets as many equal chunks as
// its length needs; each workgroup reduces its chunk to an un-normalised (m, l, O) triple per head in fp32
// and a second kernel merges the chunks (a sequence with one chunk is finished by its workgroup).  Long
// caches: the balanced form further down, one equal key range per resident workgroup and the merge inside
// the launch.
#include <mutex>
#include "common.hpp"

namespace ts {

namespace {
constexpr int kBlockKeys = 32;   // keys per wave iteration
constexpr int kMinChunk = 2048;  // chunk size aimed at when splitting is not needed to fill the chip
}

// chunks of one sequence: as few as keep every chunk within chunk_target keys (+ 1/16 slack, so
// that a cache of 2^k positions plus the token being decoded is not split for one extra key)
__host__ __device__ __forceinline__ int decode_nchunk(int len, int NCH, int chunk_target) {
  int n = (len - chunk_target / 16 + chunk_target - 1) / chunk_target;
  n = n < 1 ? 1 : n;
  return n < NCH ? n : NCH;
}

// One wave's pass over the 32-key blocks wave, wave + 4, ... of the key range [start, end) of one (sequence,
// kv head): scores, online softmax and the P.V product, leaving the wave's un-normalised state (m_run, l_run,
// o).  vst is the wave's LDS stage.  l_run comes back summed over the four lane groups.
template <int D>
__device__ __forceinline__ void decode_wave_range(const U4 (&qf)[D / 32], const ts_bf16* __restrict__ kbase,
                                                  const ts_bf16* __restrict__ vbase, int start, int end, int rot,
                                                  int wave, int lane, uint4* vst, float c_scale, float& m_run,
                                                  float& l_run, f32x4 (&o)[D / 16]) {
  constexpr int KSTEPS = D / 32;   // MFMA k-steps for Q.K
  constexpr int DT = D / 16;       // 16-wide output column tiles
  constexpr int CPR = D / 8;       // 16-byte chunks per cache row
  constexpr int VROW = CPR + 1;    // uint4 per staged V row (one pad chunk: conflict-free gathers)
  constexpr int VLOADS = kBlockKeys * CPR / 64;
  constexpr int VROW_H = VROW * 8; // staged row stride in 16-bit elements
  const int l16 = lane & 15, gq = lane >> 4;
  const uint16_t* vst_h = reinterpret_cast<const uint16_t*>(vst);
  m_run = -INFINITY;
  l_run = 0.f;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nblk = (end > start) ? (end - start + kBlockKeys - 1) / kBlockKeys : 0;
  // K and V rows are both fetched as whole rows (an instruction covers 1 KiB of consecutive bytes): only then
  // does the non-temporal hint pay (7.0 against 6.3 TB/s for a pure read; with the 16 rows x 64 bytes that an
  // MFMA operand read straight from global would touch per instruction it is 6.2).  K goes through the wave's
  // LDS stage to reach the operand layout, V follows into the same stage.
  U4 kr[VLOADS], vf[VLOADS];
  // The blocks are visited from block `rot` on, wrapping around: workgroups that start together would
  // otherwise sweep their key ranges in step, and with an unlucky distance between the ranges (the cache
  // capacity sets it) they keep landing on the same memory channels (64 x 2049 keys: 84 us at a capacity of
  // 2049 or 2176 rows, 97 us at 2064).  The order is a fixed function of the range, so results stay reproducible.
  auto block_of = [&](int j) { const int t = j + rot; return t >= nblk ? t - nblk : t; };
  auto load_block = [&](int j) {
    const int k0 = start + block_of(j) * kBlockKeys;
#pragma unroll
    for (int i = 0; i < VLOADS; ++i) {
      const int c = lane + 64 * i;
      const int key = min(k0 + c / CPR, end - 1);
      kr[i].u = ldg16_stream(kbase + (size_t)key * D + (c % CPR) * 8);
      vf[i].u = ldg16_stream(vbase + (size_t)key * D + (c % CPR) * 8);
    }
  };

  if (wave < nblk) load_block(wave);
  for (int blk = wave; blk < nblk; blk += 4) {
    const int k0 = start + block_of(blk) * kBlockKeys;
    // stage K: unpadded rows, 16-byte chunk c of row r at chunk c ^ (r % CPR) (conflict-free row writes and
    // operand reads), read it back as MFMA operands and run the score MFMAs
#pragma unroll
    for (int i = 0; i < VLOADS; ++i) {
      const int c = lane + 64 * i, r = c / CPR;
      vst[r * CPR + ((c % CPR) ^ (r & (CPR - 1)))] = kr[i].u;
    }
    __builtin_amdgcn_wave_barrier();
    U4 kf[2][KSTEPS];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      const int r = kt * 16 + l16;
#pragma unroll
      for (int j = 0; j < KSTEPS; ++j) kf[kt][j].u = vst[r * CPR + ((j * 4 + gq) ^ (r & (CPR - 1)))];
    }
    __builtin_amdgcn_wave_barrier();
    // stage V (padded rows for the 16-bit gathers below); a wave's LDS operations execute in order, so these
    // writes cannot overtake the K reads above
#pragma unroll
    for (int i = 0; i < VLOADS; ++i) {
      const int c = lane + 64 * i;
      vst[(c / CPR) * VROW + (c % CPR)] = vf[i].u;
    }
    f32x4 s[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < KSTEPS; ++j)
        s[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kt][j].b, qf[j].b, s[kt], 0, 0, 0);
    }
    if (blk + 4 < nblk) load_block(blk + 4);   // registers are free again: prefetch the next block

    // s[kt][i] = S^T[key k0 + kt*16 + gq*4 + i][head l16]
    float sv[8];
    float bm = -INFINITY;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int key = k0 + (t >> 2) * 16 + gq * 4 + (t & 3);
      sv[t] = (key < end) ? s[t >> 2][t & 3] * c_scale : -INFINITY;
      bm = fmaxf(bm, sv[t]);
    }
    bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
    bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
    const float m_new = fmaxf(m_run, bm);        // finite: the block's first key is valid
    const float alpha = exp2f(m_run - m_new);    // 0 on the first block
    float ps = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      sv[t] = exp2f(sv[t] - m_new);
      ps += sv[t];
    }
    l_run = l_run * alpha + ps;
    m_run = m_new;
    U4 pf;
#pragma unroll
    for (int t = 0; t < 4; ++t) pf.w[t] = pack_bf16(sv[2 * t], sv[2 * t + 1]);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;

    __builtin_amdgcn_wave_barrier();
    // V^T fragments: lane (dcol dt*16+l16, group gq), k-slot t <-> key (t/4)*16 + gq*4 + t%4
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      U4 vt;
#pragma unroll
      for (int t = 0; t < 8; t += 2) {
        const int key0 = (t >> 2) * 16 + gq * 4 + (t & 3);
        uint32_t lo = vst_h[key0 * VROW_H + dt * 16 + l16];
        uint32_t hi = vst_h[(key0 + 1) * VROW_H + dt * 16 + l16];
        vt.w[t >> 1] = lo | (hi << 16);
      }
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt.b, pf.b, o[dt], 0, 0, 0);
    }
    __builtin_amdgcn_wave_barrier();
  }
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
}

// The four waves' states of one key range, combined through LDS (which is reused once every wave is done with
// its stage): emit(h, col, acc, M, L) is called once per (head, column) with the un-normalised sum, the
// reference maximum and the row sum.  Ends with the LDS still holding the states: the caller puts a barrier
// before its next use.
template <int D, typename Emit>
__device__ __forceinline__ void decode_combine_waves(uint4* smem, int tid, int g, float m_run, float l_run,
                                                     const f32x4 (&o)[D / 16], Emit&& emit) {
  constexpr int DT = D / 16;
  const int lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, gq = lane >> 4;
  __syncthreads();
  float* sm_o = reinterpret_cast<float*>(smem);            // [4][16][D]
  float* sm_m = sm_o + 4 * 16 * D;                         // [4][16]
  float* sm_l = sm_m + 64;                                 // [4][16]
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
    *reinterpret_cast<f32x4*>(sm_o + ((size_t)wave * 16 + l16) * D + dt * 16 + gq * 4) = o[dt];
  if (gq == 0) {
    sm_m[wave * 16 + l16] = m_run;
    sm_l[wave * 16 + l16] = l_run;
  }
  __syncthreads();
  for (int idx = tid; idx < g * D; idx += 256) {
    const int h = idx / D, col = idx % D;
    float M = fmaxf(fmaxf(sm_m[h], sm_m[16 + h]), fmaxf(sm_m[32 + h], sm_m[48 + h]));
    float acc = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = sm_m[w * 16 + h];
      const float f = (mw == -INFINITY) ? 0.f : exp2f(mw - M);
      acc += f * sm_o[((size_t)w * 16 + h) * D + col];
      L += f * sm_l[w * 16 + h];
    }
    emit(h, col, acc, M, L);
  }
}

// Partials of the n pieces of one (sequence, head) combined in piece order, read with device-coherent loads
// (they were written by other workgroups of the same launch).
template <int D>
__device__ __forceinline__ float decode_merge_pieces_dev(const float* p, int n, int col) {
  float M = -INFINITY;
  for (int c = 0; c < n; ++c) M = fmaxf(M, ld_dev_f32(p + (size_t)c * (D + 2) + D));
  float acc = 0.f, L = 0.f;
  for (int c = 0; c < n; ++c) {
    const float mc = ld_dev_f32(p + (size_t)c * (D + 2) + D);
    const float f = (mc == -INFINITY) ? 0.f : exp2f(mc - M);
    acc += f * ld_dev_f32(p + (size_t)c * (D + 2) + col);
    L += f * ld_dev_f32(p + (size_t)c * (D + 2) + D + 1);
  }
  return acc / L;
}

template <int D>
__global__ __launch_bounds__(256) void attn_decode_split_kernel(const ts_bf16* __restrict__ q,
                                                                const ts_bf16* __restrict__ kc,
                                                                const ts_bf16* __restrict__ vc,
                                                                const int32_t* __restrict__ seq_lens,
                                                                float* __restrict__ part, int q_stride, int nq, int nkv,
                                                                int Lcap, int NCH, int chunk_target,
                                                                float c_scale /* scale * log2(e) */,
                                                                ts_bf16* __restrict__ out) {
  constexpr int KSTEPS = D / 32;   // MFMA k-steps for Q.K
  constexpr int DT = D / 16;       // 16-wide output column tiles
  constexpr int VROW = D / 8 + 1;  // uint4 per staged V row

  // (kv head, sequence) fastest, chunk slowest: consecutive workgroup ids go round-robin to the
  // 8 XCDs, and with the chunk index fastest an XCD would own fixed chunk indices, of which the
  // high ones exist only for long sequences (measured 4.5 vs 5.6 TB/s on ragged lengths).
  const int npair = gridDim.x / NCH;
  const int ch = blockIdx.x / npair, kvh = (blockIdx.x % npair) % nkv, b = (blockIdx.x % npair) / nkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, gq = lane >> 4;
  const int g = nq / nkv;
  const int len = seq_lens[b];
  if (len <= 0) {   // empty sequence: zero rows
    if (ch == 0)
      for (int idx = tid; idx < g * D; idx += 256) out[((size_t)b * nq + (size_t)kvh * g) * D + idx] = 0;
    return;
  }
  const int nchunk = decode_nchunk(len, NCH, chunk_target);
  if (ch >= nchunk) return;
  // chunks are whole 32-key blocks, spread as evenly as possible (sizes differ by one block),
  // so that the four waves of a workgroup get equal shares whenever blocks/chunk % 4 == 0
  const int nblk_total = (len + kBlockKeys - 1) / kBlockKeys;
  const int base = nblk_total / nchunk, rem = nblk_total % nchunk;
  const int start = (ch * base + min(ch, rem)) * kBlockKeys;
  const int end = min(len, start + (base + (ch < rem ? 1 : 0)) * kBlockKeys);

  extern __shared__ uint4 smem[];
  uint4* vst = smem + (size_t)wave * kBlockKeys * VROW;                  // this wave's V stage

  // Q fragments (B operand): lane (head l16, group gq) holds chunk j*4+gq of its head.
  U4 qf[KSTEPS];
  {
    const ts_bf16* qrow = q + (size_t)b * q_stride + ((size_t)kvh * g + l16) * D;
#pragma unroll
    for (int j = 0; j < KSTEPS; ++j) qf[j].u = (l16 < g) ? ldg16(qrow + (j * 4 + gq) * 8) : make_uint4(0, 0, 0, 0);
  }
  const ts_bf16* kbase = kc + ((size_t)b * nkv + kvh) * (size_t)Lcap * D;
  const ts_bf16* vbase = vc + ((size_t)b * nkv + kvh) * (size_t)Lcap * D;

  float m_run, l_run;
  f32x4 o[DT];
  const int nblk_all = (end - start + kBlockKeys - 1) / kBlockKeys;
  const int rot = nblk_all > 0 ? (int)((blockIdx.x * 2654435761u >> 8) % (unsigned)nblk_all) : 0;
  decode_wave_range<D>(qf, kbase, vbase, start, end, rot, wave, lane, vst, c_scale, m_run, l_run, o);

  // ---- merge the four waves
  decode_combine_waves<D>(smem, tid, g, m_run, l_run, o, [&](int h, int col, float acc, float M, float L) {
    if (nchunk == 1) {   // the only chunk of its sequence: final result (what the merge computes for one chunk)
      out[((size_t)b * nq + (size_t)kvh * g + h) * D + col] = f_to_bf(acc / L);
      return;
    }
    float* dst = part + (((size_t)b * nq + (size_t)kvh * g + h) * NCH + ch) * (D + 2);
    dst[col] = acc;
    if (col == 0) {
      dst[D] = M;
      dst[D + 1] = L;
    }
  });
}

// ---------------------------------------------------------------------------------------------------------
// Balanced form for long caches with mixed lengths.  With one chunk list per sequence the workgroups carry
// different amounts of work (a sequence is cut into equal chunks of at most the target, so chunk sizes range
// from half the target to the target) and their number is no multiple of what the chip holds: on the ragged
// 70B shape the last workgroups run on a half-empty chip (5.6 TB/s against 6.2 for equal lengths with the same
// total).  Here the keys of all (sequence, kv head) pairs are laid end to end in granules of 128 keys and cut
// into one equal range per workgroup, with as many workgroups as the chip holds at once; a range that crosses a
// pair boundary is processed piece by piece.  A pair cut into several pieces is combined by the last piece to
// arrive (counter per pair, partials through device-coherent accesses, pieces added in piece order), a pair
// that lies inside one range is finished by that workgroup directly.
//
// Everything is derived on the device from seq_lens, identically by every workgroup: granules per sequence,
// their prefix sums (LDS), the total, and the number of workers actually used, which is limited so that no pair
// is cut into more than NCH pieces (the partial buffer has NCH slots per pair):
//   q_min = ceil((longest sequence in granules - 1) / (NCH - 2)),  workers = min(grid, total / q_min),
// so every range has at least q_min granules and a pair of g granules spans at most (g - 1) / q_min + 2 ranges.
constexpr int kGranuleKeys = 128;       // one 32-key block for each of the four waves
constexpr int kBalancedMaxSeq = 1024;   // sequences whose prefix sums fit the kernel's LDS table

template <int D>
__global__ __launch_bounds__(256) void attn_decode_balanced_kernel(const ts_bf16* __restrict__ q,
                                                                   const ts_bf16* __restrict__ kc,
                                                                   const ts_bf16* __restrict__ vc,
                                                                   const int32_t* __restrict__ seq_lens,
                                                                   float* __restrict__ part, int q_stride, int nq,
                                                                   int nkv, int B, int Lcap, int NCH, float c_scale,
                                                                   int32_t* __restrict__ counters,
                                                                   ts_bf16* __restrict__ out) {
  constexpr int KSTEPS = D / 32;
  constexpr int DT = D / 16;
  constexpr int VROW = D / 8 + 1;
  __shared__ int s_g[kBalancedMaxSeq];     // granules of sequence b (0: empty)
  __shared__ int s_cum[kBalancedMaxSeq];   // granules of the sequences before b
  __shared__ int s_wsum[4], s_wmax[4];
  __shared__ int s_last;
  extern __shared__ uint4 smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, gq = lane >> 4;
  const int g = nq / nkv;
  uint4* vst = smem + (size_t)wave * kBlockKeys * VROW;

  // ---- granules per sequence, exclusive prefix sums, total and maximum (thread t owns sequences 4t .. 4t+3)
  for (int i = tid; i < kBalancedMaxSeq; i += 256) {
    const int len = i < B ? seq_lens[i] : 0;
    s_g[i] = len > 0 ? (len + kGranuleKeys - 1) / kGranuleKeys : 0;
  }
  __syncthreads();
  int loc[4], mine = 0, gmax = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int v = s_g[4 * tid + j];
    loc[j] = mine;
    mine += v;
    gmax = max(gmax, v);
  }
  int incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_up(incl, off, 64);
    if (lane >= off) incl += t;
    gmax = max(gmax, __shfl_xor(gmax, off, 64));
  }
  if (lane == 63) {
    s_wsum[wave] = incl;
    s_wmax[wave] = gmax;
  }
  __syncthreads();
  int before = 0;
  for (int w2 = 0; w2 < wave; ++w2) before += s_wsum[w2];
#pragma unroll
  for (int j = 0; j < 4; ++j) s_cum[4 * tid + j] = before + incl - mine + loc[j];
  const int seq_granules = s_wsum[0] + s_wsum[1] + s_wsum[2] + s_wsum[3];
  const int longest = max(max(s_wmax[0], s_wmax[1]), max(s_wmax[2], s_wmax[3]));
  __syncthreads();

  // ---- rows of empty sequences are zero; the pairs are dealt round-robin to the workgroups for this
  const int W = gridDim.x, w = blockIdx.x;
  for (int p = w; p < B * nkv; p += W) {
    const int b = p / nkv, kvh = p % nkv;
    if (s_g[b] == 0)
      for (int idx = tid; idx < g * D; idx += 256) out[((size_t)b * nq + (size_t)kvh * g) * D + idx] = 0;
  }
  const long total = (long)seq_granules * nkv;
  if (total == 0) return;
  const int q_min = max(1, (longest - 1 + (NCH - 2) - 1) / (NCH - 2));
  const int workers = (int)min((long)W, max(1L, total / q_min));
  if (w >= workers) return;
  const long per = total / workers, extra = total % workers;     // the first `extra` workers take one granule more
  const long x0 = (long)w * per + min((long)w, extra), x1 = x0 + per + (w < extra ? 1 : 0);
  auto worker_of = [&](long x) -> int {
    const long edge = extra * (per + 1);
    return (int)(x < edge ? x / (per + 1) : extra + (x - edge) / per);
  };

  // ---- the sequence that holds granule x0: the last b with nkv * s_cum[b] <= x0 (empty sequences share
  // their prefix with the non-empty one after them, which is the last of the run)
  int b;
  {
    int lo = 0, hi = B - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if ((long)s_cum[mid] * nkv <= x0) lo = mid; else hi = mid - 1;
    }
    b = __builtin_amdgcn_readfirstlane(lo);
  }
  long x = x0;
  while (x < x1) {
    const int gb = __builtin_amdgcn_readfirstlane(s_g[b]);
    const long seq0 = (long)__builtin_amdgcn_readfirstlane(s_cum[b]) * nkv;
    const int rel = (int)(x - seq0);
    const int kvh = rel / gb, gi = rel % gb;
    const long pair0 = seq0 + (long)kvh * gb;
    const long xe = min(x1, pair0 + gb);
    const int len = seq_lens[b];
    const int start = gi * kGranuleKeys;
    const int end = min(len, (gi + (int)(xe - x)) * kGranuleKeys);
    const int first = worker_of(pair0), npiece = worker_of(pair0 + gb - 1) - first + 1;
    const int piece = w - first;

    U4 qf[KSTEPS];
    {
      const ts_bf16* qrow = q + (size_t)b * q_stride + ((size_t)kvh * g + l16) * D;
#pragma unroll
      for (int j = 0; j < KSTEPS; ++j) qf[j].u = (l16 < g) ? ldg16(qrow + (j * 4 + gq) * 8) : make_uint4(0, 0, 0, 0);
    }
    const ts_bf16* kbase = kc + ((size_t)b * nkv + kvh) * (size_t)Lcap * D;
    const ts_bf16* vbase = vc + ((size_t)b * nkv + kvh) * (size_t)Lcap * D;
    float m_run, l_run;
    f32x4 o[DT];
    // (no rotated block order here: the ranges start at unrelated places of unrelated pairs already)
    decode_wave_range<D>(qf, kbase, vbase, start, end, 0, wave, lane, vst, c_scale, m_run, l_run, o);

    const size_t row0 = (size_t)b * nq + (size_t)kvh * g;
    const bool slot_ok = piece >= 0 && piece < NCH;   // holds by the choice of `workers`; never write outside the buffer
    decode_combine_waves<D>(smem, tid, g, m_run, l_run, o, [&](int h, int col, float acc, float M, float L) {
      if (npiece == 1) {
        out[(row0 + h) * D + col] = f_to_bf(acc / L);
        return;
      }
      if (!slot_ok) return;
      float* dst = part + ((row0 + h) * NCH + piece) * (D + 2);
      st_dev_f32(dst + col, acc);
      if (col == 0) {
        st_dev_f32(dst + D, M);
        st_dev_f32(dst + D + 1, L);
      }
    });
    if (npiece > 1) {
      wait_stores();
      __syncthreads();
      if (tid == 0) s_last = (atomicAdd(&counters[b * nkv + kvh], 1) == npiece - 1);
      __syncthreads();
      if (s_last) {
        for (int idx = tid; idx < g * D; idx += 256) {
          const int h = idx / D, col = idx % D;
          out[(row0 + h) * D + col] = f_to_bf(decode_merge_pieces_dev<D>(part + (row0 + h) * NCH * (D + 2), npiece, col));
        }
        if (tid == 0) __hip_atomic_store(&counters[b * nkv + kvh], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    __syncthreads();   // the LDS goes back to being the waves' stages
    x = xe;
    if (x == seq0 + (long)nkv * gb) {   // past this sequence: on to the next one that has keys
      ++b;
      while (b < B && s_g[b] == 0) ++b;
      b = __builtin_amdgcn_readfirstlane(b);
    }
  }
}

__global__ __launch_bounds__(256) void zero_words_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

template <int D>
__global__ __launch_bounds__(D) void attn_decode_merge_kernel(const float* __restrict__ part,
                                                              const int32_t* __restrict__ seq_lens,
                                                              ts_bf16* __restrict__ out, int nq, int NCH,
                                                              int chunk_target) {
  const int bh = blockIdx.x, b = bh / nq, col = threadIdx.x;
  const int len = seq_lens[b];
  ts_bf16* dst = out + (size_t)bh * D;
  if (len <= 0) {
    dst[col] = 0;
    return;
  }
  const int nchunk = decode_nchunk(len, NCH, chunk_target);
  if (nchunk == 1) return;   // written by the split kernel itself
  const float* p = part + (size_t)bh * NCH * (D + 2);
  float M = -INFINITY;
  for (int c = 0; c < nchunk; ++c) M = fmaxf(M, p[(size_t)c * (D + 2) + D]);
  float acc = 0.f, L = 0.f;
  for (int c = 0; c < nchunk; ++c) {
    const float mc = p[(size_t)c * (D + 2) + D];
    const float f = (mc == -INFINITY) ? 0.f : exp2f(mc - M);
    acc += f * p[(size_t)c * (D + 2) + col];
    L += f * p[(size_t)c * (D + 2) + D + 1];
  }
  dst[col] = f_to_bf(acc / L);
}

namespace {
struct DecodePlan {
  int NCH;            // grid extent: most chunks any sequence can have
  int chunk_target;   // keys per chunk
  bool balanced;      // equal key ranges per workgroup instead of chunks per sequence
  int pieces;         // balanced form: partial slots per (sequence, kv head)
};
// Chunks are sized from the cache capacity (lengths live on the device): about 4096 equal
// chunks if every sequence were full, but not shorter than kMinChunk keys (long chunks stream
// better: 512 workgroups of 2049 keys reach 5.6 TB/s, 2048 of 513 keys 5.3 TB/s).  A sequence
// gets a number of chunks proportional to its length, so workgroups carry similar work
// whatever the length mix (ragged 512..32768 lengths: 5.5 TB/s against 4.3 with a fixed
// number of chunks per sequence).
DecodePlan decode_plan(int B, int nkv, int Lcap) {
  DecodePlan p;
  const long total = (long)B * nkv * Lcap;
  long tgt = total / 4096;                  // ~16 chunks per CU: the last one to finish costs little
  // Long caches are cut into chunks of 4096 keys rather than 2048 as long as that still leaves four chunks
  // per CU: every extra chunk costs partial results and merge work (ragged 512..32768 lengths, 32
  // sequences: 403 us against 425 with 2176-key chunks; 1024-key chunks 483, 512-key chunks 606).
  long pref = total / 1024;
  if (pref > 2 * kMinChunk) pref = 2 * kMinChunk;
  if (pref < kMinChunk) pref = kMinChunk;
  if (tgt < pref) tgt = pref;
  tgt = (tgt + kBlockKeys * 4 - 1) / (kBlockKeys * 4) * (kBlockKeys * 4);   // whole blocks for all four waves
  p.chunk_target = (int)tgt;
  p.NCH = decode_nchunk(Lcap, 1 << 20, p.chunk_target);
  // Caches long enough for four chunks per sequence take the balanced form: a pair is then cut into pieces of
  // at least (longest sequence) / (pieces - 2) keys, sized here so that a piece of a full cache has 4096 keys.
  p.balanced = p.NCH >= 4 && B <= kBalancedMaxSeq;
  const int gcap = (Lcap + kGranuleKeys - 1) / kGranuleKeys;
  p.pieces = (gcap - 1) / (4096 / kGranuleKeys) + 2;
  if (p.pieces < 3) p.pieces = 3;
  return p;
}
size_t counter_bytes(int B, int nkv) { return round_up((size_t)B * nkv * sizeof(int32_t), 256); }

// workgroups the chip holds at once (two per CU at this kernel's register count)
int resident_workgroups() {
  static int cached[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 512;
  if (cached[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    cached[dev] = 2 * cus;
  }
  return cached[dev];
}
}  // namespace

// Split-KV partials; in the balanced form also room for the arrival counters of a caller that brings none.
size_t attention_decode_workspace_bytes(int B, int nq, int nkv, int d, int Lcap) {
  if (B <= 0 || nq <= 0 || nkv <= 0 || d <= 0 || Lcap <= 0) return 0;
  const DecodePlan p = decode_plan(B, nkv, Lcap);
  if (p.balanced) return round_up((size_t)B * nq * p.pieces * (d + 2) * sizeof(float), 256) + counter_bytes(B, nkv);
  return (size_t)B * nq * p.NCH * (d + 2) * sizeof(float);
}

int launch_attention_decode(const ts_bf16* q, int q_stride, const ts_bf16* kc, const ts_bf16* vc, const int32_t* seq_lens,
                            ts_bf16* out, int B, int nq, int nkv, int d, int Lcap, float scale, void* ws,
                            size_t ws_bytes, hipStream_t s, int32_t* counters) {
  if (B == 0) return TS_OK;
  const DecodePlan plan = decode_plan(B, nkv, Lcap);
  const int NCH = plan.NCH;
  const size_t need = attention_decode_workspace_bytes(B, nq, nkv, d, Lcap);
  TS_REQUIRE(ws != nullptr && ws_bytes >= need, TS_ERR_WORKSPACE,
             "ts_attention_decode: workspace %zu bytes < required %zu", ws_bytes, need);
  const float c_scale = scale * 1.4426950408889634f;
  float* part = reinterpret_cast<float*>(ws);
  if (plan.balanced) {
    // a caller without counters of its own (the stand-alone entry points) gets them from the end of the
    // workspace, zeroed by a launch of their own; the layer's counters are zeroed by its first kernel
    if (counters == nullptr) {
      counters = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(ws) + need - counter_bytes(B, nkv));
      TS_LAUNCH("zero_words", zero_words_kernel, dim3(cdiv(B * nkv, 256)), dim3(256), 0, s, counters, B * nkv);
      TS_LAUNCH_CHECK("zero_words");
    }
    dim3 grid_b((unsigned)resident_workgroups());
    if (d == 128) {
      const size_t stage = (size_t)4 * kBlockKeys * 17 * sizeof(uint4);
      const size_t merge = (size_t)(4 * 16 * 128 + 128) * sizeof(float);
      TS_LAUNCH_LAST("attn_decode_split", attn_decode_balanced_kernel<128>, grid_b, dim3(256), stage > merge ? stage : merge, s,
                     q, kc, vc, seq_lens, part, q_stride, nq, nkv, B, Lcap, plan.pieces, c_scale, counters, out);
    } else {
      const size_t stage = (size_t)4 * kBlockKeys * 9 * sizeof(uint4);
      const size_t merge = (size_t)(4 * 16 * 64 + 128) * sizeof(float);
      TS_LAUNCH_LAST("attn_decode_split", attn_decode_balanced_kernel<64>, grid_b, dim3(256), stage > merge ? stage : merge, s,
                     q, kc, vc, seq_lens, part, q_stride, nq, nkv, B, Lcap, plan.pieces, c_scale, counters, out);
    }
    TS_LAUNCH_CHECK("attn_decode_balanced");
    return TS_OK;
  }
  // Chunks per sequence: with one chunk the split kernel writes the result itself, else a merge kernel follows.
  dim3 grid((unsigned)NCH * nkv * B);
  const bool merge_kernel = NCH > 1;
  if (d == 128) {
    const size_t stage = (size_t)4 * kBlockKeys * 17 * sizeof(uint4);
    const size_t merge = (size_t)(4 * 16 * 128 + 128) * sizeof(float);
    const size_t smem = stage > merge ? stage : merge;
    TS_LAUNCH_EX(!merge_kernel, "attn_decode_split", attn_decode_split_kernel<128>, grid, dim3(256), smem, s, q, kc, vc, seq_lens, part, q_stride, nq,
                       nkv, Lcap, NCH, plan.chunk_target, c_scale, out);
    TS_LAUNCH_CHECK("attn_decode_split");
    if (merge_kernel)
      TS_LAUNCH_LAST("attn_decode_merge", attn_decode_merge_kernel<128>, dim3(B * nq), dim3(128), 0, s, part, seq_lens, out, nq, NCH, plan.chunk_target);
  } else {
    const size_t stage = (size_t)4 * kBlockKeys * 9 * sizeof(uint4);
    const size_t merge = (size_t)(4 * 16 * 64 + 128) * sizeof(float);
    const size_t smem = stage > merge ? stage : merge;
    TS_LAUNCH_EX(!merge_kernel, "attn_decode_split", attn_decode_split_kernel<64>, grid, dim3(256), smem, s, q, kc, vc, seq_lens, part, q_stride, nq,
                       nkv, Lcap, NCH, plan.chunk_target, c_scale, out);
    TS_LAUNCH_CHECK("attn_decode_split");
    if (merge_kernel)
      TS_LAUNCH_LAST("attn_decode_merge", attn_decode_merge_kernel<64>, dim3(B * nq), dim3(64), 0, s, part, seq_lens, out, nq, NCH, plan.chunk_target);
  }
  TS_LAUNCH_CHECK("attn_decode_merge");
  return TS_OK;
}

// ---- the entry point that allocates nothing: split-KV partials in a file-scope device array ---------------
// Each GPU the library runs on holds its own copy of the array, at its own address, until the process ends.
// In host code the array's name is only a stand-in for the symbol: the device address is looked up once per
// device (with that device current) and kept; everything on the host uses the looked-up pointer.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
  int dev = -1;
  TS_HIP(hipGetDevice(&dev));
  TS_REQUIRE(dev >= 0 && dev < kMaxDevices, TS_ERR_UNSUPPORTED_SHAPE, "ts_attention_decode_static: device index %d", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* found = nullptr;
    TS_HIP(hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)));
    TS_REQUIRE(found != nullptr, TS_ERR_HIP, "ts_attention_decode_static: no device address for the scratch array");
    g_scratch_ptr[dev] = found;
  }
  *out = g_scratch_ptr[dev];
  return TS_OK;
}
}  // namespace

}  // namespace ts

extern "C" {

size_t ts_attention_decode_static_limit(void) { return ts::kStaticScratchBytes; }

int ts_attention_decode_static(const ts_bf16* q, const ts_bf16* kcache, const ts_bf16* vcache, const int32_t* seq_lens,
                               ts_bf16* out, int B, int nq, int nkv, int d, int Lcap, float scale, void* stream) {
  using namespace ts;
  TS_REQUIRE(B >= 0 && nq > 0 && nkv > 0 && d > 0 && Lcap > 0, TS_ERR_INVALID_ARG,
             "ts_attention_decode_static: B=%d nq=%d nkv=%d d=%d Lcap=%d", B, nq, nkv, d, Lcap);
  TS_REQUIRE(nq % nkv == 0, TS_ERR_INVALID_ARG, "ts_attention_decode_static: nq %% nkv != 0");
  TS_REQUIRE(B == 0 || (q && kcache && vcache && seq_lens && out), TS_ERR_INVALID_ARG, "ts_attention_decode_static: null pointer");
  TS_REQUIRE(aligned16(q) && aligned16(kcache) && aligned16(vcache) && aligned16(out), TS_ERR_INVALID_ARG,
             "ts_attention_decode_static: pointer not 16-byte aligned");
  TS_REQUIRE(d == 64 || d == 128, TS_ERR_UNSUPPORTED_SHAPE, "ts_attention_decode_static: d=%d (64 or 128 supported)", d);
  TS_REQUIRE(nq / nkv <= 16, TS_ERR_UNSUPPORTED_SHAPE, "ts_attention_decode_static: GQA group %d > 16", nq / nkv);
  if (B == 0) return TS_OK;
  const size_t need = attention_decode_workspace_bytes(B, nq, nkv, d, Lcap);
  TS_REQUIRE(need <= kStaticScratchBytes, TS_ERR_WORKSPACE,
             "ts_attention_decode_static: split-KV partials need %zu bytes, the built-in scratch holds %zu "
             "(use ts_attention_decode with a workspace of your own)", need, kStaticScratchBytes);
  void* ptr = nullptr;
  int rc = static_scratch(&ptr);
  if (rc != TS_OK) return rc;
  // What has to start at zero, the arrival counters of the balanced form at the end of the array, is cleared by a
  // small kernel that the launch function enqueues itself; every partial a merge reads was written by this call.
  return launch_attention_decode(q, nq * d, kcache, vcache, seq_lens, out, B, nq, nkv, d, Lcap, scale, ptr,
                                 kStaticScratchBytes, reinterpret_cast<hipStream_t>(stream), nullptr);
}

}  // extern "C"
