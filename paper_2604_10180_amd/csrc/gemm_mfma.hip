// Compute-bound bf16 projection C = A * W^T (+ residual) for thousands of token rows: the
// prefill regime of Sec. 2.3, where the matrix cores and not HBM set the time.
//
// One workgroup = 8 waves (two per SIMD, so one wave's LDS/global traffic hides behind the
// other's MFMAs) computes a 256 (n) x 256 (m) tile of C; wave (wn, wm) owns 128 n x 64 m as
// 8 x 4 accumulators of the 16x16x32 MFMA (on random operands a register-resident loop of this
// shape sustains 2.05 PFLOP/s under the chip's power management against 1.83 for 32x32x16).
// K advances 64 per step through a two-stage LDS ring that is filled by direct global->LDS
// loads (no VGPR round trip, no LDS store instructions).
//
// LDS tile layout: row r (one W row or one token row) holds its 64 k-values as 8 chunks of
// 16 bytes, 128 bytes per row, no padding (a direct load writes lane i's 16 bytes at
// base + 16 i, so padding is not available).  Bank conflicts are avoided by a swizzle that
// is applied on the GLOBAL side: the lane that fills physical chunk p of row r fetches
// logical chunk p ^ f(r), f(r) = (r & 7) ^ ((r >> 3) & 1).  Eight consecutive lanes fetch
// one whole 128-byte row (fully coalesced), and an MFMA operand read (16 rows x four logical
// chunks) touches every bank group equally.
//
// What bounds it (8192 x 28672 x 4096): power.  With all-zero operands (full clock) the kernel runs at
// 1.69 PFLOP/s: 2.0 without its ring loads, 1.79 when every load hits L2, and the L2 warm-up below closes most
// of the gap to that (1.47 without it).  With random operands every structural variant lands at 1.2-1.3
// (1.81 without the ring loads, 1.34 with L2 hits only): the matrix cores, the fragment reads, the L2->LDS
// stream and the L2 misses each take their share of a fixed power budget, and the clock drops to 1.8 GHz.
// The vendor library (same 256 x 256 x 64 tile, same MFMA shape) reaches 1.39-1.43 there and 2.14 on zeros.
// Four-wave variants (128 x 128 per wave; also with a four-stage ring of 32-wide K steps and partial vmcnt
// waits) passed parity and measured 1.08-1.12 on random data.
//
// Epilogue: the residual tile is staged into LDS coalesced, each lane adds its accumulators to
// its own slots in fp32 and rounds once, and the bf16 tile leaves as full 512-byte row
// segments.
#include "common.hpp"
#include <type_traits>

namespace ts {

namespace {

constexpr int kTile = 256;
constexpr int kBK = 64;
constexpr int kStageU4 = 2 * kTile * kBK * 2 / 16;   // W tile + A tile = 64 KiB = 4096 uint4

typedef __attribute__((address_space(3))) void lds_void;

// The two ring stages are separate LDS variables on purpose: the compiler then knows that a
// direct load into one stage cannot alias operand reads from the other, and does not make
// those reads wait for the loads in flight.
__shared__ uint4 g_stage0[kStageU4];
__shared__ uint4 g_stage1[kStageU4];

__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0) only
// Workgroup barrier without the counter waits that __syncthreads() adds (it would wait for every load in
// flight): the caller has waited for exactly what the ring needs.
__device__ __forceinline__ void ring_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

}  // namespace

// GLU = true is the gate/up projection of a SwiGLU MLP with the activation applied in the epilogue: W holds F
// gate rows followed by F up rows (N = 2F); a tile then covers 128 gate columns and the 128 up columns of
// the same hidden units, writes both to C as usual and silu(gate) * up, computed from the bf16-rounded values
// exactly as the stand-alone kernel does, to act [M, F].  Requires F % 128 == 0; no residual.
template <bool GLU>
__device__ __forceinline__ void gemm_mfma256_body(const ts_bf16* __restrict__ A, const ts_bf16* __restrict__ W,
                                                  const ts_bf16* __restrict__ residual, ts_bf16* __restrict__ C, int M,
                                                  int N, int K, int tiles_m, int tiles_n, ts_bf16* __restrict__ act) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave & 1, wm = wave >> 1;

  // Workgroup -> tile.  Consecutive workgroup ids go round-robin to the 8 XCDs (each with its
  // own L2), so ids are first regrouped so that an XCD works on a contiguous run of logical
  // tiles; logical tiles walk groups of 8 row tiles down the columns, so the tiles an XCD runs
  // at a time form a compact patch that shares operand tiles in that L2.
  int lid = blockIdx.x;
  const int nblocks = gridDim.x;
  if ((nblocks & 7) == 0) lid = (lid & 7) * (nblocks >> 3) + (lid >> 3);
  constexpr int GM = 8;
  const int per_group = GM * tiles_n;
  const int first_m = (lid / per_group) * GM;
  const int gsz = min(GM, tiles_m - first_m);
  const int tile_m = first_m + (lid % per_group) % gsz, tile_n = (lid % per_group) / gsz;
  const int F = N >> 1;                                   // GLU only
  const int mb = tile_m * kTile, nb = tile_n * (GLU ? kTile / 2 : kTile);

  // ---- global -> LDS assignment: load q of wave w fills LDS rows (q*8 + w)*8 .. +8 of a tile;
  // lane i lands at 16 i inside that 1 KiB, i.e. row i/8, physical chunk i%8.
  const int lrow = lane >> 3;
  const int cl = (lane & 7) ^ lrow ^ (wave & 1);            // logical chunk this lane fetches
  const char* wtile = reinterpret_cast<const char*>(W + (size_t)nb * K);
  const char* atile = reinterpret_cast<const char*>(A + (size_t)mb * K);
  uint32_t woff[4], aoff[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int R = q * 64 + wave * 8 + lrow;
    // GLU: tile rows 128..255 are the up rows of the same 128 hidden units
    const int wr = GLU ? (R < 128 ? R : F + R - 128) : min(R, N - 1 - nb);
    woff[q] = (uint32_t)wr * (uint32_t)K * 2u + cl * 16;
    aoff[q] = (uint32_t)min(R, M - 1 - mb) * (uint32_t)K * 2u + cl * 16;
  }
  // L2 warm-up.  The 32 workgroups an XCD runs at a time form a patch of 8 row tiles x 4 column tiles, so every
  // operand line is wanted by 8 (W) or 4 (A) workgroups at about the same K step and exactly one of them takes
  // the L2 miss.  Each workgroup therefore touches, three K steps ahead, its share of the patch's lines: 32 of
  // its 256 W rows (chosen by its row-tile index in the patch) and 64 of its 256 A rows (by its column-tile
  // index), 12 lanes per wave, 4 bytes each.  Purely a hint: correctness does not depend on which
  // workgroups really run together.
  const char* pfbase;
  {
    const int pidx = wave * 12 + min(lane, 11);
    const int jm = tile_m - first_m, cn = tile_n & 3;
    if (pidx < 32) {
      const int R = jm * 32 + pidx;
      const int wr = GLU ? (R < 128 ? R : F + R - 128) : min(R, N - 1 - nb);
      pfbase = wtile + (size_t)wr * K * 2;
    } else {
      pfbase = atile + (size_t)min(cn * 64 + pidx - 32, M - 1 - mb) * K * 2;
    }
  }
  // The loaded word is only kept alive until the wait that covers it (an ordinary register load, so the
  // compiler's own counter bookkeeping stays exact); lanes 12..63 repeat lane 11's address.
  uint32_t warm_prev = 0;
  auto warm_l2 = [&](int k0) -> uint32_t {
    return *reinterpret_cast<const uint32_t*>(pfbase + (size_t)k0 * 2);
  };
  // load pair h (0..3) of a K step: one W and one A instruction of this wave
  auto issue_pair = [&](uint4* stage, int k0, int h) {
    uint4* sb = stage + wave * 64 + h * 512;
    __builtin_amdgcn_global_load_lds(wtile + woff[h] + (size_t)k0 * 2, (lds_void*)sb, 16, 0, 0);
    __builtin_amdgcn_global_load_lds(atile + aoff[h] + (size_t)k0 * 2, (lds_void*)(sb + 2048), 16, 0, 0);
  };

  // ---- operand fragments of the 16x16x32 MFMA: lane (r16, kq) supplies row r16 and the 8 k-values of 16-byte
  // chunk kq of a 32-wide k-slice, for both operands (which 8 k-values a chunk holds is free as long as both
  // agree).  16 rows x 128 bytes = 2048 bytes per fragment; the swizzle depends on the row only through r16.
  const int r16 = lane & 15, kq = lane >> 4;
  const int f = (r16 & 7) ^ (r16 >> 3);
  // lane groups kq and kq + 2 (lanes l and l + 32) are served together by the LDS: their chunks must differ in the
  // lowest bit, or the swizzle sends the two to the same banks (measured: half of all LDS cycles in conflict)
  const int kperm = ((kq & 1) << 1) | (kq >> 1);
  int frag_off[2];
#pragma unroll
  for (int sl = 0; sl < 2; ++sl) frag_off[sl] = r16 * 128 + (((sl * 4 + kperm) ^ f) * 16);
  const int wbase = wn * 128 * 128;
  const int abase = 32768 + wm * 64 * 128;

  // acc[i][j]: output columns n = i*16 .. +16 (8 blocks), token rows m = j*16 .. +16 (4 blocks) of the wave tile
  f32x4 acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  // A K step of 64 is four units of 16 MFMAs: (k-slice sl, column half h) = 4 W fragments x the 4 A fragments
  // of the slice.  Fragments of the next unit are read from LDS while the current unit multiplies.
  auto load_w = [&](const char* st, int sl, int h, U4(&wf)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      wf[i].u = *reinterpret_cast<const uint4*>(st + wbase + (h * 4 + i) * 2048 + frag_off[sl]);
  };
  auto load_a = [&](const char* st, int sl, U4(&af)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) af[j].u = *reinterpret_cast<const uint4*>(st + abase + j * 2048 + frag_off[sl]);
  };
  auto mfma16 = [&](auto hc, const U4(&wf)[4], const U4(&af)[4]) {
    constexpr int h = decltype(hc)::value;
    // serpentine walk: one operand changes from one MFMA to the next (2 % more sustained on random operands
    // than a row-major walk in a register-resident loop: less switching on the operand buses)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int j = (i & 1) ? 3 - jj : jj;
        acc[h * 4 + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i].b, af[j].b, acc[h * 4 + i][j], 0, 0, 0);
      }
  };
  // instruction order of the unit just written: MFMA, (LDS read, MFMA) x R, the remaining MFMAs
  auto order = [&](auto rc) {
    constexpr int R = decltype(rc)::value;
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 15 - R, 0);
  };
  using H0 = std::integral_constant<int, 0>;
  using H1 = std::integral_constant<int, 1>;
  using R4 = std::integral_constant<int, 4>;
  using R8 = std::integral_constant<int, 8>;
  // The last unit of a stage (slice 1, half 1) is read before the barrier that ends the stage and multiplied
  // after it, next to the first fragment reads of the following stage: the matrix cores have work while
  // those reads are in flight.  (wB, aB) carry it; zero before the first step.
  const int nk = K / kBK;
  const int klast = (nk - 1) * kBK;
  U4 wA[4], wB[4], aA[4], aB[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) wB[i].u = aB[i].u = make_uint4(0, 0, 0, 0);
  auto step = [&](const uint4* cur, uint4* nxt, int knext) {
    const char* st = reinterpret_cast<const char*>(cur);
#pragma unroll
    for (int h = 0; h < 4; ++h) issue_pair(nxt, knext, h);
    __builtin_amdgcn_sched_barrier(0);
    const uint32_t warm = warm_l2(min(knext + 2 * kBK, klast));   // issued last: the wait below leaves it in flight
    __builtin_amdgcn_sched_barrier(0);   // keep the loads ahead of the MFMAs they overlap with
    load_a(st, 0, aA);
    load_w(st, 0, 0, wA);
    mfma16(H1{}, wB, aB);                 // slice 1, half 1 of the previous stage
    order(R8{});
    __builtin_amdgcn_sched_barrier(0);
    load_w(st, 0, 1, wB);
    mfma16(H0{}, wA, aA);
    order(R4{});
    __builtin_amdgcn_sched_barrier(0);
    load_a(st, 1, aB);
    load_w(st, 1, 0, wA);
    mfma16(H1{}, wB, aA);
    order(R8{});
    __builtin_amdgcn_sched_barrier(0);
    load_w(st, 1, 1, wB);
    mfma16(H0{}, wA, aB);
    order(R4{});
    __builtin_amdgcn_sched_barrier(0);
    // the next stage has landed (all but the newest load, the warm-up) and this one is fully read
    __builtin_amdgcn_s_waitcnt(0x0071);
    ring_barrier();
    asm volatile("" ::"v"(warm_prev));   // the previous step's warm-up word has arrived by now
    warm_prev = warm;
  };
  // Every step prefetches; the last one re-fetches the final K slice into the stage nobody
  // reads any more (cheaper than a second, load-free copy of the step), and its loads have
  // landed before the epilogue reuses the ring.
#pragma unroll
  for (int h = 0; h < 4; ++h) issue_pair(g_stage0, 0, h);
  wait_vm0();
  __syncthreads();
  int it = 0;
  for (; it + 2 <= nk; it += 2) {
    step(g_stage0, g_stage1, (it + 1) * kBK);
    step(g_stage1, g_stage0, min((it + 2) * kBK, klast));
  }
  if (it < nk) step(g_stage0, g_stage1, klast);   // odd number of K steps
  mfma16(H1{}, wB, aB);
  asm volatile("" ::"v"(warm_prev));   // keeps the last step's warm-up load, which its wait counts on
  wait_vm0();   // no load may still be in flight towards LDS when the ring is reused and the workgroup ends

  // ---- epilogue.  The ring is dead; the two stages now hold the bf16 image of the C tile:
  // rows 0..127 in stage 0, 128..255 in stage 1, 512 bytes per row, unpadded.  Logical 16-byte
  // chunk ch of row m sits at physical chunk ch ^ (m & 15), and its two 8-byte halves are
  // swapped when m & 16: the 32 lanes that write one accumulator register quad (32 different
  // rows, one column group) then cover all banks once.
  auto image_row = [&](int m) -> char* {
    return reinterpret_cast<char*>((m & 128) ? g_stage1 : g_stage0) + (m & 127) * 512;
  };
  auto swap_halves = [](uint4 v) { return make_uint4(v.z, v.w, v.x, v.y); };
  if (residual != nullptr) {
    // stage the residual tile, coalesced: thread -> (row p*16 + tid/32, physical chunk tid%32)
#pragma unroll 4
    for (int p = 0; p < 16; ++p) {
      const int m = p * 16 + (tid >> 5), pc = tid & 31;
      const int ch = pc ^ (m & 15);
      const int gm = min(mb + m, M - 1), gn = min(nb + ch * 8, N - 8);
      uint4 v = ldg16(residual + (size_t)gm * N + gn);
      if (m & 16) v = swap_halves(v);
      *reinterpret_cast<uint4*>(image_row(m) + pc * 16) = v;
    }
    __syncthreads();
  }
  // acc[i][j][e] is D[n = i*16 + kq*4 + e][m = j*16 + r16] of the wave tile; every 8-byte slot of the image
  // is read (residual) and written by exactly one lane.
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int m = wm * 64 + j * 16 + r16;
    char* row = image_row(m);
    const int hoff = ((kq & 1) ^ ((m >> 4) & 1)) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int ch = wn * 16 + i * 2 + (kq >> 1);
      uint2* slot = reinterpret_cast<uint2*>(row + ((ch ^ (m & 15)) * 16) + hoff);
      float v0 = acc[i][j][0], v1 = acc[i][j][1], v2 = acc[i][j][2], v3 = acc[i][j][3];
      if (residual != nullptr) {
        const uint2 r = *slot;
        v0 += bf_lo(r.x); v1 += bf_hi(r.x); v2 += bf_lo(r.y); v3 += bf_hi(r.y);
      }
      uint2 o;
      o.x = pack_bf16(v0, v1);
      o.y = pack_bf16(v2, v3);
      *slot = o;
    }
  }
  __syncthreads();
#pragma unroll 4
  for (int p = 0; p < 16; ++p) {
    const int m = p * 16 + (tid >> 5), pc = tid & 31;
    const int ch = pc ^ (m & 15);
    const int gm = mb + m;
    const int gn = GLU ? (ch < 16 ? nb + ch * 8 : F + nb + (ch - 16) * 8) : nb + ch * 8;
    uint4 v = *reinterpret_cast<const uint4*>(image_row(m) + pc * 16);
    if (m & 16) v = swap_halves(v);
    if (gm < M && gn < N) stg16(C + (size_t)gm * N + gn, v);
  }
  if (GLU) {
    // act[m, nb + 8c .. +8) = silu(gate) * up from image chunks c and 16 + c of row m (the swizzle only
    // permutes the low four bits of the chunk index, so the pair sits at pc and 16 + pc)
#pragma unroll 4
    for (int p = 0; p < 8; ++p) {
      const int m = p * 32 + (tid >> 4), c = tid & 15;
      const int pc = c ^ (m & 15);
      U4 gv, uv, o;
      gv.u = *reinterpret_cast<const uint4*>(image_row(m) + pc * 16);
      uv.u = *reinterpret_cast<const uint4*>(image_row(m) + (16 + pc) * 16);
      if (m & 16) {
        gv.u = swap_halves(gv.u);
        uv.u = swap_halves(uv.u);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float g0 = bf_lo(gv.w[j]), g1 = bf_hi(gv.w[j]);
        const float a0 = g0 / (1.0f + __expf(-g0)) * bf_lo(uv.w[j]);
        const float a1 = g1 / (1.0f + __expf(-g1)) * bf_hi(uv.w[j]);
        o.w[j] = pack_bf16(a0, a1);
      }
      if (mb + m < M) stg16(act + (size_t)(mb + m) * F + nb + c * 8, o.u);
    }
  }
}

__global__ __launch_bounds__(512) void gemm_mfma256_kernel(const ts_bf16* __restrict__ A, const ts_bf16* __restrict__ W,
                                                           const ts_bf16* __restrict__ residual,
                                                           ts_bf16* __restrict__ C, int M, int N, int K, int tiles_m,
                                                           int tiles_n) {
  gemm_mfma256_body<false>(A, W, residual, C, M, N, K, tiles_m, tiles_n, nullptr);
}

__global__ __launch_bounds__(512) void gemm_mfma256_glu_kernel(const ts_bf16* __restrict__ A,
                                                               const ts_bf16* __restrict__ W,
                                                               ts_bf16* __restrict__ gate_up,
                                                               ts_bf16* __restrict__ act, int M, int N, int K,
                                                               int tiles_m, int tiles_n) {
  gemm_mfma256_body<true>(A, W, nullptr, gate_up, M, N, K, tiles_m, tiles_n, act);
}

bool gemm_mfma256_supported(int M, int N, int K) {
  // full 64-wide K steps, 16-byte output chunks, tile-relative byte offsets within 32 bits
  return K >= kBK && K % kBK == 0 && N % 8 == 0 && N >= 8 && (long)K * 2 * kTile < (1L << 31);
}

bool gemm_mfma256_glu_supported(int M, int F, int K) {
  // more token rows than the streaming kernel takes and enough 256 x 256 tiles (the conditions under which
  // the plain projection runs on this kernel), whole 128-column halves, byte offsets of the up rows relative
  // to the tile within 32 bits
  return M > 128 && (long)cdiv(M, kTile) * cdiv(2 * F, kTile) >= 192 && K >= kBK && K % kBK == 0 && F >= 128 &&
         F % 128 == 0 && ((long)F + 256) * K * 2 < (1L << 32);
}

int launch_gemm_mfma256_glu(const ts_bf16* A, const ts_bf16* W, ts_bf16* gate_up, ts_bf16* act, int M, int F, int K,
                            hipStream_t s) {
  const int tiles_m = cdiv(M, kTile), tiles_n = F / 128;
  TS_LAUNCH_LAST("gemm_mfma256_glu", gemm_mfma256_glu_kernel, dim3(tiles_m * tiles_n), dim3(512), 0, s, A, W, gate_up, act, M,
            2 * F, K, tiles_m, tiles_n);
  TS_LAUNCH_CHECK("gemm_mfma256_glu");
  return TS_OK;
}

int launch_gemm_mfma256(const ts_bf16* A, const ts_bf16* W, const ts_bf16* residual, ts_bf16* C, int M, int N, int K,
                        hipStream_t s) {
  const int tiles_m = cdiv(M, kTile), tiles_n = cdiv(N, kTile);
  TS_LAUNCH_LAST("gemm_mfma256", gemm_mfma256_kernel, dim3(tiles_m * tiles_n), dim3(512), 0, s, A, W, residual, C, M, N, K,
            tiles_m, tiles_n);
  TS_LAUNCH_CHECK("gemm_mfma256");
  return TS_OK;
}

}  // namespace ts
