// Compute-bound bf16 projection C = A * W^T (+ residual) for thousands of token rows: the
// prefill regime of Sec. 2.3, where the matrix cores and not HBM set the time.
//
// One workgroup = 8 waves (two per SIMD, so one wave's LDS/global traffic hides behind the
// other's MFMAs) computes a 256 (n) x 256 (m) tile of C; wave (wn, wm) owns 128 n x 64 m as
// 4 x 2 accumulators of the 32x32x16 MFMA.  K advances 64 per step through a two-stage LDS
// ring that is filled by direct global->LDS loads (no VGPR round trip, no LDS store
// instructions).
//
// LDS tile layout: row r (one W row or one token row) holds its 64 k-values as 8 chunks of
// 16 bytes, 128 bytes per row, no padding (a direct load writes lane i's 16 bytes at
// base + 16 i, so padding is not available).  Bank conflicts are avoided by a swizzle that
// is applied on the GLOBAL side: the lane that fills physical chunk p of row r fetches
// logical chunk p ^ f(r), f(r) = (r & 7) ^ ((r >> 3) & 1).  Eight consecutive lanes fetch
// one whole 128-byte row (fully coalesced), and an MFMA operand read (32 rows x one logical
// chunk) touches every bank group equally.
//
// What bounds it (8192 x 28672 x 4096): with random operands the chip is power-managed (1.81 GHz against
// 2.19 GHz without the ring loads) and every variant with real loads lands at 1.2 PFLOP/s; the vendor library
// reaches 1.42-1.52 there.  With all-zero operands (full clock) this kernel runs at 1.38, at 1.96 without its
// loads, 1.70 when every load hits L2 and 1.67 without the ring barrier: the 19 % of the loads that miss L2
// arrive late and unevenly and the barrier couples all eight waves to the slowest.  Four-wave variants
// (128 x 128 per wave; also with a four-stage ring of 32-wide K steps and partial vmcnt waits) passed parity
// and measured 1.08-1.12 on random data.
//
// Epilogue: the residual tile is staged into LDS coalesced, each lane adds its accumulators to
// its own slots in fp32 and rounds once, and the bf16 tile leaves as full 512-byte row
// segments.
#include "common.hpp"

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
  const int r32 = lane & 31, g = lane >> 5;
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
  // load pair h (0..3) of a K step: one W and one A instruction of this wave
  auto issue_pair = [&](uint4* stage, int k0, int h) {
    uint4* sb = stage + wave * 64 + h * 512;
    __builtin_amdgcn_global_load_lds(wtile + woff[h] + (size_t)k0 * 2, (lds_void*)sb, 16, 0, 0);
    __builtin_amdgcn_global_load_lds(atile + aoff[h] + (size_t)k0 * 2, (lds_void*)(sb + 2048), 16, 0, 0);
  };

  // ---- operand fragment addresses: row base + swizzled chunk for k-step ks
  const int f = (r32 & 7) ^ ((r32 >> 3) & 1);
  int frag_off[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) frag_off[ks] = r32 * 128 + (((ks * 2) ^ g ^ f) * 16);
  const int wbase = wn * 128 * 128;
  const int abase = 32768 + wm * 64 * 128;

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // One K step.  Operand fragments are double buffered in registers: the LDS reads for k-step
  // ks+1 are issued before the 8 MFMAs of ks and interleaved with them one to one.  The eight
  // direct loads that fill the other stage are issued first, so that they have the whole step
  // to land (spreading them over the step measured slower).
  auto load_frags = [&](const char* st, int ks, U4(&wf)[4], U4(&af)[2]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) wf[i].u = *reinterpret_cast<const uint4*>(st + wbase + i * 4096 + frag_off[ks]);
#pragma unroll
    for (int j = 0; j < 2; ++j) af[j].u = *reinterpret_cast<const uint4*>(st + abase + j * 4096 + frag_off[ks]);
  };
  auto mfma8 = [&](const U4(&wf)[4], const U4(&af)[2]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i].b, af[j].b, acc[i][j], 0, 0, 0);
  };
  auto order = [&]() {   // instruction order of the block just written: MFMA, (LDS read, MFMA) x 6, MFMA
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
#pragma unroll
    for (int r = 0; r < 6; ++r) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
  };
  auto step = [&](const uint4* cur, uint4* nxt, int knext) {
    const char* st = reinterpret_cast<const char*>(cur);
#pragma unroll
    for (int h = 0; h < 4; ++h) issue_pair(nxt, knext, h);
    __builtin_amdgcn_sched_barrier(0);   // keep the loads ahead of the MFMAs they overlap with
    U4 wf0[4], af0[2], wf1[4], af1[2];
    load_frags(st, 0, wf0, af0);
    __builtin_amdgcn_sched_barrier(0);
    load_frags(st, 1, wf1, af1);
    mfma8(wf0, af0);
    order();
    __builtin_amdgcn_sched_barrier(0);
    load_frags(st, 2, wf0, af0);
    mfma8(wf1, af1);
    order();
    __builtin_amdgcn_sched_barrier(0);
    load_frags(st, 3, wf1, af1);
    mfma8(wf0, af0);
    order();
    __builtin_amdgcn_sched_barrier(0);
    mfma8(wf1, af1);
    wait_vm0();
    __syncthreads();
  };
  // Every step prefetches; the last one re-fetches the final K slice into the stage nobody
  // reads any more (cheaper than a second, load-free copy of the step), and its loads have
  // landed before the epilogue reuses the ring.
  const int nk = K / kBK;
  const int klast = (nk - 1) * kBK;
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
  // acc[i][j][e] is D[n = i*32 + (e/4)*8 + g*4 + e%4][m = j*32 + r32] of the wave tile; every
  // 8-byte slot of the image is read (residual) and written by exactly one lane.
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int m = wm * 64 + j * 32 + r32;
    char* row = image_row(m);
    const int hoff = (g ^ ((m >> 4) & 1)) * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int gi = 0; gi < 4; ++gi) {
        const int ch = wn * 16 + i * 4 + gi;
        uint2* slot = reinterpret_cast<uint2*>(row + ((ch ^ (m & 15)) * 16) + hoff);
        float v0 = acc[i][j][gi * 4 + 0], v1 = acc[i][j][gi * 4 + 1], v2 = acc[i][j][gi * 4 + 2],
              v3 = acc[i][j][gi * 4 + 3];
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
  TS_LAUNCH("gemm_mfma256_glu", gemm_mfma256_glu_kernel, dim3(tiles_m * tiles_n), dim3(512), 0, s, A, W, gate_up, act, M,
            2 * F, K, tiles_m, tiles_n);
  TS_LAUNCH_CHECK("gemm_mfma256_glu");
  return TS_OK;
}

int launch_gemm_mfma256(const ts_bf16* A, const ts_bf16* W, const ts_bf16* residual, ts_bf16* C, int M, int N, int K,
                        hipStream_t s) {
  const int tiles_m = cdiv(M, kTile), tiles_n = cdiv(N, kTile);
  TS_LAUNCH("gemm_mfma256", gemm_mfma256_kernel, dim3(tiles_m * tiles_n), dim3(512), 0, s, A, W, residual, C, M, N, K,
            tiles_m, tiles_n);
  TS_LAUNCH_CHECK("gemm_mfma256");
  return TS_OK;
}

}  // namespace ts
