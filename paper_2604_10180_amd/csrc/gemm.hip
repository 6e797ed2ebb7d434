// bf16 projections C = A * W^T on the gfx950 matrix cores.
//
// Two kernels, because the paper's regime split (Sec. 2.3) applies to the very same
// product: with a handful of rows the weights are streamed once from HBM and the kernel is
// bandwidth-bound ("skinny", also used per expert by the grouped MoE product); with
// thousands of rows it is MFMA-bound ("tiled").
//
// Both use W as the MFMA "A" operand (rows = output columns n) and the activations as the
// "B" operand (columns = token rows m), so each lane ends up with 4 consecutive n of one
// token row and stores 8 contiguous bytes.  Both operands are K-contiguous in memory, so a
// lane's 8-element operand fragment is one 16-byte load; which 8 k-values a lane group
// holds is free as long as both operands agree, and is chosen for contiguous loads.
#include <type_traits>
#include "common.hpp"

namespace ts {

// ============================================================================ skinny
struct SkinnyArgs {
  const ts_bf16* A;
  const int32_t* row_map;
  int row_div;
  const ts_bf16* W;
  const int32_t* offsets;   // grouped only
  const ts_bf16* residual;
  void* C;                  // bf16 or f32 [M,N]
  float* partial;           // [S,M,N] when S > 1
  int M, N, K;
  int kslice, S;
  int f32out;
  long w_group_stride;      // elements between experts
};

// Workgroup: WAVES waves (4, 7 or 8); wave w owns 16*NT rows of W; the activation k-slab [MT*16, 128] is
// staged in LDS and shared by all waves (the first four stage it).  K advances 128 per iteration; for MFMA
// step j lane (r, g) of a wave (r = lane%16, g = lane/16) holds the 8 k-values of 16-byte chunk j*4+g of W row
// r and of the token row it multiplies.  From 33 token rows on the W fragments are loaded straight from
// global in that layout (a row's four lanes read 64 contiguous bytes per load); up to 32 rows W is fetched as
// whole cache lines and rearranged through a per-wave LDS stage (see WSTAGE below).
// WAVES = 7 exists because the number of workgroups should be a multiple of the 256 CUs (a CU's bandwidth is
// capped, so 448 workgroups take as long as 512 would): 28672 output columns are 256 x 112.
template <int MT, int NT, bool GROUPED, int NS, int WAVES = 4>
__global__ __launch_bounds__(64 * WAVES) void gemm_skinny_kernel(SkinnyArgs a) {
  constexpr int ROWS = MT * 16;
  constexpr int D = NS - 1;    // prefetch distance in 128-wide K slabs
  // activation slabs in LDS: the D the ring needs where the W stage shares the LDS, else one per register stage
  // (stage indices are then compile-time constants)
  constexpr int AST = (MT <= 2) ? D : NS;
  constexpr int LDS_ROW = 17;  // uint4 per staged row: 16 data + 1 pad (272 B stride, conflict-free b128 reads)
  extern __shared__ uint4 smem[];
  uint4(*lds)[ROWS][LDS_ROW] = reinterpret_cast<uint4(*)[ROWS][LDS_ROW]>(smem);
  // behind the activation ring, per wave, a W stage of 16 rows x 8 chunks (half a slab), chunk c of row r at
  // chunk c ^ (r & 7) ^ (r >> 3) (conflict-free whole-line writes and operand reads), reused for every half

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  uint4* wst = smem + AST * ROWS * LDS_ROW + wave * 128;
  int row0 = 0, Mtot = a.M;
  const ts_bf16* W = a.W;
  if (GROUPED) {
    const int e = blockIdx.z;
    row0 = a.offsets[e];
    Mtot = a.offsets[e + 1] - row0;
    if (Mtot <= 0) return;
    W += (size_t)e * a.w_group_stride;
  }
  const int N = a.N, K = a.K;
  const int nbase = blockIdx.x * (16 * NT * WAVES) + wave * (16 * NT);
  const int kbeg = blockIdx.y * a.kslice;
  const int kend = min(K, kbeg + a.kslice);

  // W is fetched as whole cache lines (load i of a 16-row block: lane takes chunk lane % 8 of line i / 2 of
  // row 8 (i % 2) + lane / 8, so an instruction covers eight whole 128-byte lines): only in that form does
  // the non-temporal hint pay (7.0 against 6.3 TB/s for a pure read stream; with 16 rows x 64 bytes per
  // instruction, which is what reading MFMA operands straight from global amounts to, it costs 3 %).  The
  // wave's LDS stage turns each half slab into operand fragments.
  constexpr bool WSTAGE = MT <= 2;
  const ts_bf16* wrow[NT][WSTAGE ? 4 : 1];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if constexpr (WSTAGE) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int n = min(nbase + nt * 16 + 8 * (i & 1) + (lane >> 3), N - 1);
        wrow[nt][i] = W + (size_t)n * K + (8 * (i >> 1) + (lane & 7)) * 8;
      }
    } else {
      int n = min(nbase + nt * 16 + l16, N - 1);
      wrow[nt][0] = W + (size_t)n * K + g * 8;
    }
  }
  const int st_r = tid >> 4, st_c = tid & 15;  // staging: row st_r + 16*i, chunk st_c

  for (int m0 = 0; m0 < Mtot; m0 += ROWS) {
    const int Mcur = min(ROWS, Mtot - m0);
    const ts_bf16* arow[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int r = st_r + 16 * i;
      long src = (long)row0 + m0 + (r < Mcur ? r : 0);   // rows past the end re-read row 0
      if (a.row_map != nullptr) src = a.row_map[src] / a.row_div;
      arow[i] = a.A + (size_t)src * K;
    }
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // NS-stage ring, prefetch distance D = NS-1: while slab `it` is multiplied, the W fragments
    // of slabs it+1 .. it+D are in flight in registers and the activation slab it+D-1 moves
    // from registers to LDS.  One barrier per slab; barriers wait on LDS only, never on the
    // outstanding global loads.
    U4 wbuf[NS][NT][4], areg[MT];

    // Rows past the end of A or W are clamped to a valid row: they only feed output elements
    // that are never stored.  Only a K tail (K % 128 != 0) needs zeros, and zeroing the W
    // fragment is enough (the matching A chunk is re-read from the last valid chunk of the
    // same row).  Full slabs use unpredicated loads so nothing consumes a load at issue time.
    auto load_w = [&](int k0, U4(&dst)[NT][4]) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          dst[nt][j].u = WSTAGE ? ldg16_stream(wrow[nt][WSTAGE ? j : 0] + k0) : ldg16(wrow[nt][0] + k0 + j * 32);
    };
    auto load_w_tail = [&](int k0, U4(&dst)[NT][4]) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int lo = (WSTAGE ? 8 * (j >> 1) + (lane & 7) : g) * 8;   // lane offset held in the pointer
          const int k = WSTAGE ? k0 : k0 + j * 32;
          const bool ok = k + lo < kend;
          dst[nt][j].u = ldg16_or_zero(wrow[nt][WSTAGE ? j : 0] + (ok ? k : kbeg - lo), ok);
        }
    };
    auto load_a = [&](int k0) {
      if (WAVES > 4 && tid >= 256) return;
      const int k = min(k0 + st_c * 8, kend - 8);
#pragma unroll
      for (int i = 0; i < MT; ++i) areg[i].u = ldg16(arow[i] + k);
    };
    auto store_a = [&](int buf) {
      if (WAVES > 4 && tid >= 256) return;
#pragma unroll
      for (int i = 0; i < MT; ++i) lds[buf][st_r + 16 * i][st_c] = areg[i].u;
    };
    auto compute = [&](int buf, U4(&wraw)[NT][4]) {
      // slab lines -> operand fragments through the wave's stage, half a slab at a time: fragment j of lane
      // (l16, g) is chunk j*4 + g of row l16.  A wave's LDS operations execute in order, so the next half's
      // writes cannot overtake these reads.
      U4 w[NT][4];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        if constexpr (WSTAGE) {
#pragma unroll
          for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
              const int r = 8 * ii + (lane >> 3);
              wst[r * 8 + ((lane & 7) ^ (r & 7) ^ (r >> 3))] = wraw[nt][2 * h + ii].u;
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
              w[nt][2 * h + jj].u = wst[l16 * 8 + ((jj * 4 + g) ^ (l16 & 7) ^ (l16 >> 3))];
            __builtin_amdgcn_wave_barrier();
          }
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) w[nt][j] = wraw[nt][j];
        }
      }
      // read a whole k-step of activation fragments before the MFMAs that use them, so the
      // LDS latency is paid once per step instead of once per MFMA
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        U4 b[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) b[mt].u = lds[buf][mt * 16 + l16][j * 4 + g];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[nt][j].b, b[mt].b, acc[mt][nt], 0, 0, 0);
      }
    };

    // Full 128-wide slabs run through the ring.  Workgroups start their K walk at different
    // slabs (and wrap around), so that they do not all sweep the same activation addresses
    // and the same HBM channels in step.
    const int nfull = (kend - kbeg) / 128;
    if (nfull > 0) {
      const int rot = (int)((blockIdx.x * 7u + blockIdx.z * 3u) % (unsigned)nfull);
      auto slab = [&](int it) { int r = it + rot; return kbeg + (r >= nfull ? r - nfull : r) * 128; };
      // one ring step; CHECKED = false is the branch-free steady state
      auto step = [&](auto checked, auto stage, int it) {
        constexpr bool CHECKED = decltype(checked)::value;
        constexpr int u = decltype(stage)::value;
        if (!CHECKED || it + D - 1 < nfull) store_a(WSTAGE ? (it + D - 1) % AST : (u + D - 1) % NS);
        if (!CHECKED || it + D < nfull) {
          const int kn = slab(it + D);
          load_a(kn);
          load_w(kn, wbuf[(u + D) % NS]);
        }
        compute(WSTAGE ? it % AST : u, wbuf[u]);
        __syncthreads();
      };
      using T_ = std::true_type;
      using F_ = std::false_type;
      // prologue: slabs 0 .. D-2 go all the way into LDS, slab D-1 stays in registers
#pragma unroll
      for (int p = 0; p < D; ++p) {
        if (p < nfull) {
          load_a(slab(p));
          load_w(slab(p), wbuf[p]);
          if (p < D - 1) store_a(p);
        }
      }
      __syncthreads();
      int it = 0;
      for (; it + 2 * NS - 2 < nfull; it += NS) {
        step(F_{}, std::integral_constant<int, 0>{}, it);
        step(F_{}, std::integral_constant<int, 1>{}, it + 1);
        step(F_{}, std::integral_constant<int, 2>{}, it + 2);
        if constexpr (NS > 3) step(F_{}, std::integral_constant<int, 3>{}, it + 3);
      }
      for (; it < nfull; it += NS) {
        step(T_{}, std::integral_constant<int, 0>{}, it);
        if (it + 1 < nfull) step(T_{}, std::integral_constant<int, 1>{}, it + 1);
        if (it + 2 < nfull) step(T_{}, std::integral_constant<int, 2>{}, it + 2);
        if constexpr (NS > 3) {
          if (it + 3 < nfull) step(T_{}, std::integral_constant<int, 3>{}, it + 3);
        }
      }
    }
    if (kbeg + nfull * 128 < kend) {   // K tail: one partial slab, not pipelined
      const int kt = kbeg + nfull * 128;
      load_a(kt);
      load_w_tail(kt, wbuf[0]);
      store_a(0);
      __syncthreads();
      compute(0, wbuf[0]);
      __syncthreads();
    }

    // epilogue: lane holds D[n = g*4+i][m = l16] for every (mt, nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int ml = mt * 16 + l16;
      if (ml >= Mcur) continue;
      const size_t orow = (size_t)row0 + m0 + ml;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int n = nbase + nt * 16 + g * 4;
        if (n >= N) continue;
        f32x4 v = acc[mt][nt];
        if (a.S > 1) {
          float* p = a.partial + ((size_t)blockIdx.y * a.M + orow) * N + n;
          if ((N & 3) == 0) {
            *reinterpret_cast<f32x4*>(p) = v;
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (n + i < N) p[i] = v[i];
          }
          continue;
        }
        const size_t o = orow * N + n;
        if (a.f32out) {
          float* p = reinterpret_cast<float*>(a.C) + o;
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (n + i < N) p[i] = v[i];
          continue;
        }
        ts_bf16* cp = reinterpret_cast<ts_bf16*>(a.C) + o;
        if ((N & 3) == 0) {
          if (a.residual != nullptr) {
            uint2 r = *reinterpret_cast<const uint2*>(a.residual + o);
            v[0] += bf_lo(r.x); v[1] += bf_hi(r.x); v[2] += bf_lo(r.y); v[3] += bf_hi(r.y);
          }
          uint2 out;
          out.x = pack_bf16(v[0], v[1]);
          out.y = pack_bf16(v[2], v[3]);
          *reinterpret_cast<uint2*>(cp) = out;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (n + i < N) {
              float x = v[i];
              if (a.residual != nullptr) x += bf_to_f(a.residual[o + i]);
              cp[i] = f_to_bf(x);
            }
        }
      }
    }
  }
}

// out[m,n] = sum_s partial[s,m,n] (+ residual), slices added in ascending s (deterministic).  A thread owns two
// consecutive elements of the flattened [M*N] result; the loads of four slices are in flight together (the
// slices are independent addresses, a loop of dependent loads would pay the memory latency S times).  An odd
// element count (possible only for an fp32 result with odd N) leaves a last single element.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial,
                                                            const ts_bf16* __restrict__ residual, void* C, long MN,
                                                            int S, int f32out) {
  const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 2;
  if (i >= MN) return;
  if (i + 1 >= MN) {   // odd tail
    float a0 = 0.f;
    for (int s = 0; s < S; ++s) a0 += partial[(size_t)s * MN + i];
    if (f32out) reinterpret_cast<float*>(C)[i] = a0;
    else reinterpret_cast<ts_bf16*>(C)[i] = f_to_bf(residual != nullptr ? a0 + bf_to_f(residual[i]) : a0);
    return;
  }
  const bool even = (MN & 1) == 0;   // rows keep 8-byte alignment only then
  auto ld2 = [&](int s) {
    const float* p = partial + (size_t)s * MN + i;
    return even ? *reinterpret_cast<const float2*>(p) : make_float2(p[0], p[1]);
  };
  float a0 = 0.f, a1 = 0.f;
  int s = 0;
  for (; s + 4 <= S; s += 4) {
    const float2 p0 = ld2(s), p1 = ld2(s + 1), p2 = ld2(s + 2), p3 = ld2(s + 3);
    a0 += p0.x; a1 += p0.y;
    a0 += p1.x; a1 += p1.y;
    a0 += p2.x; a1 += p2.y;
    a0 += p3.x; a1 += p3.y;
  }
  for (; s < S; ++s) {
    const float2 p = ld2(s);
    a0 += p.x;
    a1 += p.y;
  }
  if (f32out) {
    float* c = reinterpret_cast<float*>(C) + i;
    c[0] = a0;
    c[1] = a1;
    return;
  }
  if (residual != nullptr) {   // bf16 results have an even N (checked at the boundary): pairs are 4-byte aligned
    uint32_t r = *reinterpret_cast<const uint32_t*>(residual + i);
    a0 += bf_lo(r);
    a1 += bf_hi(r);
  }
  *reinterpret_cast<uint32_t*>(reinterpret_cast<ts_bf16*>(C) + i) = pack_bf16(a0, a1);
}

// ============================================================================ tiled
// Block tile BM (token rows) x BN (W rows), BK = 64, 4 waves as 2 (n) x 2 (m); every wave
// computes (BN/2) x (BM/2) with 32x32x16 MFMAs.  Both operand tiles go global -> registers
// -> LDS (144-byte row stride: conflict-free 16-byte operand reads), double buffered, one
// barrier per K step.
template <int BM, int BN, bool F32OUT>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(const ts_bf16* __restrict__ A, const ts_bf16* __restrict__ W,
                                                         const ts_bf16* __restrict__ residual, void* __restrict__ C,
                                                         int M, int N, int K, int tiles_m, int tiles_n,
                                                         float* __restrict__ partial, int kslice) {
  constexpr int TN = BN / 64, TM = BM / 64;
  // split-K: blockIdx.y owns K range [kbeg, kend) and writes an fp32 partial tile (partial != nullptr)
  const int kbeg = blockIdx.y * kslice, kend = min(K, kbeg + kslice);
  constexpr int LW = BN / 32, LA = BM / 32;  // 16-byte chunks per thread per tile
  extern __shared__ uint4 smem[];
  // layout: [2][BN][9] then [2][BM][9]
  uint4(*sW)[BN][9] = reinterpret_cast<uint4(*)[BN][9]>(smem);
  uint4(*sA)[BM][9] = reinterpret_cast<uint4(*)[BM][9]>(smem + 2 * BN * 9);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r32 = lane & 31, g = lane >> 5;
  const int wn = wave & 1, wm = wave >> 1;
  // Workgroup -> tile.  Consecutive workgroup ids go round-robin to the 8 XCDs (each with its
  // own L2), so ids are first regrouped so that an XCD works on a contiguous run of logical
  // tiles; logical tiles walk groups of 8 row tiles down the columns, so the ~32 tiles an XCD
  // runs at a time form an 8 x 4 patch that shares operand tiles in that L2.
  int lid = blockIdx.x;
  const int nblocks = gridDim.x;
  if ((nblocks & 7) == 0) lid = (lid & 7) * (nblocks >> 3) + (lid >> 3);
  constexpr int GM = 8;
  const int per_group = GM * tiles_n;
  const int first_m = (lid / per_group) * GM;
  const int gsz = min(GM, tiles_m - first_m);
  const int tile_m = first_m + (lid % per_group) % gsz, tile_n = (lid % per_group) / gsz;
  const int mb = tile_m * BM, nb = tile_n * BN;

  const int st_r = tid >> 3, st_c = tid & 7;
  const ts_bf16* wptr[LW];
  const ts_bf16* aptr[LA];
#pragma unroll
  for (int i = 0; i < LW; ++i) wptr[i] = W + (size_t)min(nb + st_r + 32 * i, N - 1) * K + st_c * 8;
#pragma unroll
  for (int i = 0; i < LA; ++i) aptr[i] = A + (size_t)min(mb + st_r + 32 * i, M - 1) * K + st_c * 8;

  f32x16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 wr[LW], ar[LA];
  auto gload = [&](int k0) {
    if (k0 + 64 <= kend) {   // full K step: plain loads, nothing consumes them at issue time
#pragma unroll
      for (int i = 0; i < LW; ++i) wr[i] = ldg16(wptr[i] + k0);
#pragma unroll
      for (int i = 0; i < LA; ++i) ar[i] = ldg16(aptr[i] + k0);
    } else {
      const bool ok = (k0 + st_c * 8) < kend;
      const int kk = ok ? k0 : kbeg;
#pragma unroll
      for (int i = 0; i < LW; ++i) wr[i] = ldg16_or_zero(wptr[i] + kk, ok);
#pragma unroll
      for (int i = 0; i < LA; ++i) ar[i] = ldg16_or_zero(aptr[i] + kk, ok);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LW; ++i) sW[buf][st_r + 32 * i][st_c] = wr[i];
#pragma unroll
    for (int i = 0; i < LA; ++i) sA[buf][st_r + 32 * i][st_c] = ar[i];
  };

  gload(kbeg);
  sstore(0);
  __syncthreads();
  int it = 0;
  for (int k0 = kbeg; k0 < kend; k0 += 64, ++it) {
    const int cur = it & 1;
    const bool more = (k0 + 64) < kend;
    if (more) gload(k0 + 64);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      U4 wf[TN], af[TM];
#pragma unroll
      for (int i = 0; i < TN; ++i) wf[i].u = sW[cur][wn * (BN / 2) + i * 32 + r32][ks * 2 + g];
#pragma unroll
      for (int j = 0; j < TM; ++j) af[j].u = sA[cur][wm * (BM / 2) + j * 32 + r32][ks * 2 + g];
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i].b, af[j].b, acc[i][j], 0, 0, 0);
    }
    if (more) sstore(cur ^ 1);
    __syncthreads();
  }

  // epilogue: acc[i][j][e] is D[n = (e/4)*8 + g*4 + e%4][m = r32] of the 32x32 tile
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int m = mb + wm * (BM / 2) + j * 32 + r32;
    if (m >= M) continue;
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
      for (int gi = 0; gi < 4; ++gi) {
        const int n = nb + wn * (BN / 2) + i * 32 + gi * 8 + g * 4;
        if (n >= N) continue;
        float v[4] = {acc[i][j][gi * 4 + 0], acc[i][j][gi * 4 + 1], acc[i][j][gi * 4 + 2], acc[i][j][gi * 4 + 3]};
        const size_t o = (size_t)m * N + n;
        if (partial != nullptr) {
          float* p = partial + (size_t)blockIdx.y * M * N + o;
          if ((N & 3) == 0) {
            *reinterpret_cast<f32x4*>(p) = f32x4{v[0], v[1], v[2], v[3]};
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n + e < N) p[e] = v[e];
          }
          continue;
        }
        if (F32OUT) {
          float* p = reinterpret_cast<float*>(C) + o;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < N) p[e] = v[e];
        } else {
          ts_bf16* cp = reinterpret_cast<ts_bf16*>(C) + o;
          if ((N & 3) == 0) {
            if (residual != nullptr) {
              uint2 r = *reinterpret_cast<const uint2*>(residual + o);
              v[0] += bf_lo(r.x); v[1] += bf_hi(r.x); v[2] += bf_lo(r.y); v[3] += bf_hi(r.y);
            }
            uint2 out;
            out.x = pack_bf16(v[0], v[1]);
            out.y = pack_bf16(v[2], v[3]);
            *reinterpret_cast<uint2*>(cp) = out;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n + e < N) {
                float x = v[e];
                if (residual != nullptr) x += bf_to_f(residual[o + e]);
                cp[e] = f_to_bf(x);
              }
          }
        }
      }
    }
  }
}

// ============================================================================ host side
namespace {

constexpr int kSkinnyMaxM = 128;
// A handful of output columns (the MoE router): the weight matrix is a few rows, so the
// streaming kernel (looping over row blocks of A) beats one tile of the MFMA-bound kernel.
constexpr int kSkinnyMaxN = 16;
inline bool use_skinny(int M, int N) { return M <= kSkinnyMaxM || N <= kSkinnyMaxN; }

struct SkinnyPlan {
  int NT, S, kslice;
  int waves = 4;
};

// Launch shape of the streaming kernel.  128-row workgroups halve the activation re-reads,
// but only pay when there are at least as many of them as CUs (a CU keeps a bounded number of
// cache misses in flight, so an idle CU is lost bandwidth); otherwise 64-row workgroups, split
// along K until there are about two per CU.
SkinnyPlan plan_skinny(int M, int N, int K) {
  SkinnyPlan p;
  const int t2 = cdiv(N, 128), t1 = cdiv(N, 64);
  p.S = 1;
  if (t2 >= 256) {
    p.NT = 2;
  } else {
    p.NT = 1;
    if (t1 < 448) {
      int want = cdiv(512, t1);
      int maxs = K / 512;  // keep at least four 128-wide K steps per slice
      if (maxs < 1) maxs = 1;
      p.S = want < maxs ? want : maxs;
      if (p.S > 16) p.S = 16;
    }
  }
  // Up to 64 token rows: also consider seven- and eight-wave workgroups (112 / 128 weight rows) and, from 33
  // rows on, every form the kernel has.
  if (M <= 32 && p.NT == 1) {   // (very wide outputs already stream at the cap with 128-row workgroups)
    // The most loaded CU runs ceil(workgroups / 256) of them, a workgroup's traffic is its weight slice plus
    // the activation rows it re-reads from L2 (about a third as expensive per byte), every K slice adds
    // partial-sum traffic, and at equal width the wide forms measured a tenth faster.  Measured with it: 70B
    // shapes at 32 rows, qkv 46 -> 36 us, o 40 -> 31 us; at 8 rows qkv 42 -> 34 us, o 39 -> 29 us.
    const int rows = M <= 16 ? 16 : 32;
    auto score = [&](int waves, int NT, int S) {
      const int cols = 16 * waves * NT;
      const long wgs = (long)cdiv(N, cols) * S;
      const double quant = (double)((wgs + 255) / 256 * 256) / (double)wgs;
      return quant * (1.0 + 0.35 * rows / cols) * (1.0 + 0.02 * S) * (waves > 4 ? 0.9 : 1.0);
    };
    const double legacy = score(4, p.NT, p.S);
    double best = legacy;
    int maxs = K / 512;
    maxs = maxs < 1 ? 1 : (maxs > 16 ? 16 : maxs);
    for (int waves : {7, 8})
      for (int S = 1; S <= maxs && N >= 16 * waves; ++S) {
        const double sc = score(waves, 1, S);
        if (sc < 0.95 * legacy && sc < best) {
          best = sc;
          p.waves = waves;
          p.NT = 1;
          p.S = S;
        }
      }
  } else if (M <= 64 && p.NT == 1) {
    // 33 to 64 rows: every form (4, 7 or 8 waves x 16 or 32 weight rows per wave x 1..16 K slices) is scored in
    // bytes through the most loaded CU: workgroups on that CU x (the workgroup's weight slice + its activation
    // rows at half the cost per byte + 40 KB for filling and draining its ring) + the fp32 partials of a K
    // split, written and read back, at 1.5 x the cost per byte.  The constants are a fit to a sweep of all
    // forms over the projection shapes of the 8B and 70B layers; at 64 rows the choice is the best form measured
    // for all four 8B shapes (qkv 24.5 -> 22.9 us and o 20.9 -> 18.3 us including their reduce kernels, by
    // using four K slices instead of five and eight; 8B decode layer 0.2245 -> 0.2204 ms).  Up to 32 rows
    // the same fit is 2 % faster kernel by kernel and 1 % slower on the pipelined step, where two projections
    // share the chip and its fewer, fatter workgroups pack worse; the rule above stays there.
    auto score = [&](int waves, int NT, int S) {
      const int cols = 16 * waves * NT;
      const int kslice = (int)round_up((size_t)cdiv(K, S), 128);
      const int slices = cdiv(K, kslice);
      const long wgs = (long)cdiv(N, cols) * slices;
      double t = (double)((wgs + 255) / 256) * ((double)kslice * 2.0 * (cols + 0.5 * 64) + 40e3);
      if (slices > 1) t += 2.0 * M * (double)N * 4.0 * slices / 256.0 * 1.5;
      return t;
    };
    const double legacy = score(4, p.NT, p.S);
    double best = legacy;
    int maxs = K / 512;
    maxs = maxs < 1 ? 1 : (maxs > 16 ? 16 : maxs);
    for (int waves : {4, 7, 8})
      for (int NT : {1, 2})
        for (int S = 1; S <= maxs && N >= 16 * waves * NT; ++S) {
          if ((long)cdiv(N, 16 * waves * NT) * S < 128) continue;   // at least half the CUs
          const double sc = score(waves, NT, S);
          if (sc < 0.97 * legacy && sc < best) {
            best = sc;
            p.waves = waves;
            p.NT = NT;
            p.S = S;
          }
        }
  }
  p.kslice = (int)round_up((size_t)cdiv(K, p.S), 128);
  p.S = cdiv(K, p.kslice);
  return p;
}

// Kernels that need more than the default dynamic-LDS limit raise it once.
template <typename KernelT>
void allow_lds(KernelT kernel, size_t bytes) {
  if (bytes > 48 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)bytes);
}

// Ring depth: four stages (three slabs of W in flight per wave) for up to 32 token rows, where
// it measured faster; three stages otherwise (the fourth costs occupancy at 64 rows).
template <int MT, int NT> constexpr int skinny_stages() { return (MT <= 2 && NT == 1) ? 4 : 3; }

template <int MT, bool GROUPED>
void launch_skinny_mt(const SkinnyArgs& a, int NT, dim3 grid, hipStream_t s, int waves = 4) {
  if constexpr ((!GROUPED && MT <= 4) || (GROUPED && MT >= 4)) {
    if (waves == 7 || waves == 8) {
      auto go = [&](auto nt_c, auto w_c) {
        constexpr int NTc = decltype(nt_c)::value, Wc = decltype(w_c)::value;
        constexpr int NS = skinny_stages<MT, NTc>();
        const size_t smem = ((size_t)(MT <= 2 ? NS - 1 : NS) * MT * 16 * 17 + (MT <= 2 ? Wc * 128 : 0)) * sizeof(uint4);
        allow_lds(gemm_skinny_kernel<MT, NTc, GROUPED, NS, Wc>, smem);
        TS_LAUNCH_EX(a.S == 1, "gemm_skinny", (gemm_skinny_kernel<MT, NTc, GROUPED, NS, Wc>), grid, dim3(64 * Wc), smem, s, a);
      };
      using I1 = std::integral_constant<int, 1>;
      using I2 = std::integral_constant<int, 2>;
      using I7 = std::integral_constant<int, 7>;
      using I8 = std::integral_constant<int, 8>;
      if (waves == 7) { if (NT == 2) go(I2{}, I7{}); else go(I1{}, I7{}); }
      else { if (NT == 2) go(I2{}, I8{}); else go(I1{}, I8{}); }
      return;
    }
  }
  if (NT == 2) {
    constexpr int NS = skinny_stages<MT, 2>();
    const size_t smem = ((size_t)(MT <= 2 ? NS - 1 : NS) * MT * 16 * 17 + (MT <= 2 ? 4 * 128 : 0)) * sizeof(uint4);
    allow_lds(gemm_skinny_kernel<MT, 2, GROUPED, NS>, smem);
    TS_LAUNCH_EX(a.S == 1, "gemm_skinny", (gemm_skinny_kernel<MT, 2, GROUPED, NS>), grid, dim3(256), smem, s, a);
  } else {
    constexpr int NS = skinny_stages<MT, 1>();
    const size_t smem = ((size_t)(MT <= 2 ? NS - 1 : NS) * MT * 16 * 17 + (MT <= 2 ? 4 * 128 : 0)) * sizeof(uint4);
    allow_lds(gemm_skinny_kernel<MT, 1, GROUPED, NS>, smem);
    TS_LAUNCH_EX(a.S == 1, "gemm_skinny", (gemm_skinny_kernel<MT, 1, GROUPED, NS>), grid, dim3(256), smem, s, a);
  }
}

template <bool GROUPED>
void launch_skinny(const SkinnyArgs& a, int mrows, int NT, dim3 grid, hipStream_t s, int waves = 4) {
  if (mrows <= 16) launch_skinny_mt<1, GROUPED>(a, NT, grid, s, waves);
  else if (mrows <= 32) launch_skinny_mt<2, GROUPED>(a, NT, grid, s, waves);
  else if (mrows <= 64) launch_skinny_mt<4, GROUPED>(a, NT, grid, s, waves);
  else if (mrows <= 96) launch_skinny_mt<6, GROUPED>(a, NT, grid, s, waves);
  else launch_skinny_mt<8, GROUPED>(a, NT, grid, s, waves);
}

}  // namespace

// Split of the 128 x 128-tile kernel along K for projections of a few hundred rows (a large
// decode batch): 2 x 48 tiles leave most CUs idle and the weight stream at a fifth of the HBM
// rate.  Slices until there are about 384 workgroups (512 measured slower); each slice keeps at least 512 of K.
int plan_tiled_split(int M, int N, int K) {
  const long tiles = (long)cdiv(M, 128) * cdiv(N, 128);
  if (tiles >= 192) return 1;
  int S = (int)((384 + tiles - 1) / tiles);
  const int maxs = K / 512;
  if (S > maxs) S = maxs;
  if (S > 16) S = 16;
  return S < 1 ? 1 : S;
}

template <int BM, int BN>
int launch_tiled(const ts_bf16* A, const ts_bf16* W, const ts_bf16* residual, void* C, bool f32out, int M, int N, int K,
                 hipStream_t s, int S = 1, float* partial = nullptr) {
  const int tiles_m = cdiv(M, BM), tiles_n = cdiv(N, BN);
  const size_t smem = (size_t)2 * (BM + BN) * 9 * sizeof(uint4);
  const int kslice = (int)round_up((size_t)cdiv(K, S), 64);
  S = cdiv(K, kslice);
  if (S == 1) partial = nullptr;
  dim3 grid(tiles_m * tiles_n, S);
  if (f32out) {
    allow_lds(gemm_tiled_kernel<BM, BN, true>, smem);
    TS_LAUNCH_EX(partial == nullptr, "gemm_tiled", (gemm_tiled_kernel<BM, BN, true>), grid, dim3(256), smem, s, A, W, residual, C, M, N, K,
              tiles_m, tiles_n, partial, kslice);
  } else {
    allow_lds(gemm_tiled_kernel<BM, BN, false>, smem);
    TS_LAUNCH_EX(partial == nullptr, "gemm_tiled", (gemm_tiled_kernel<BM, BN, false>), grid, dim3(256), smem, s, A, W, residual, C, M, N, K,
              tiles_m, tiles_n, partial, kslice);
  }
  TS_LAUNCH_CHECK("gemm_tiled");
  if (partial != nullptr) {
    const long MN = (long)M * N;
    TS_LAUNCH_LAST("splitk_reduce", splitk_reduce_kernel, dim3((unsigned)(((MN + 1) / 2 + 255) / 256)), dim3(256), 0, s, partial,
              residual, C, MN, S, f32out ? 1 : 0);
    TS_LAUNCH_CHECK("splitk_reduce");
  }
  return TS_OK;
}

// the tiled 128 x 128 path is taken when neither the streaming kernel nor 256 x 256 tiles apply
static bool use_tiled128(int M, int N) { return !use_skinny(M, N) && (long)cdiv(M, 256) * cdiv(N, 256) < 192; }

size_t gemm_workspace_bytes(int M, int N, int K) {
  if (M <= 0 || N <= 0 || K <= 0) return 0;
  if (use_tiled128(M, N)) {
    const int S = plan_tiled_split(M, N, K);
    return S > 1 ? (size_t)S * M * N * sizeof(float) : 0;
  }
  if (!use_skinny(M, N)) return 0;
  SkinnyPlan p = plan_skinny(M, N, K);
  return p.S > 1 ? (size_t)p.S * M * N * sizeof(float) : 0;
}

int launch_gemm(const ts_bf16* A, const ts_bf16* W, const ts_bf16* residual, void* C, bool f32out, int M, int N, int K,
                void* ws, size_t ws_bytes, hipStream_t s) {
  if (M == 0) return TS_OK;
  if (use_skinny(M, N)) {
    SkinnyPlan p = plan_skinny(M, N, K);
    const size_t need = p.S > 1 ? (size_t)p.S * M * N * sizeof(float) : 0;
    TS_REQUIRE(need == 0 || (ws != nullptr && ws_bytes >= need), TS_ERR_WORKSPACE,
               "ts_gemm_bf16: workspace %zu bytes < required %zu", ws_bytes, need);
    SkinnyArgs a{};
    a.A = A; a.row_map = nullptr; a.row_div = 1; a.W = W; a.offsets = nullptr; a.residual = residual; a.C = C;
    a.partial = reinterpret_cast<float*>(ws); a.M = M; a.N = N; a.K = K; a.kslice = p.kslice; a.S = p.S;
    a.f32out = f32out ? 1 : 0; a.w_group_stride = 0;
    dim3 grid(cdiv(N, 16 * p.waves * p.NT), p.S, 1);
    launch_skinny<false>(a, M, p.NT, grid, s, p.waves);
    TS_LAUNCH_CHECK("gemm_skinny");
    if (p.S > 1) {
      long MN = (long)M * N;
      TS_LAUNCH_LAST("splitk_reduce", splitk_reduce_kernel, dim3((unsigned)(((MN + 1) / 2 + 255) / 256)), dim3(256), 0, s,
                         reinterpret_cast<const float*>(ws), residual, C, MN, p.S, f32out ? 1 : 0);
      TS_LAUNCH_CHECK("splitk_reduce");
    }
    return TS_OK;
  }
  // 256 x 256 tiles when they still give every CU work (direct-to-LDS kernel when the shape
  // allows it), 128 x 128 tiles otherwise.
  if ((long)cdiv(M, 256) * cdiv(N, 256) >= 192) {
    if (!f32out && gemm_mfma256_supported(M, N, K))
      return launch_gemm_mfma256(A, W, residual, reinterpret_cast<ts_bf16*>(C), M, N, K, s);
    return launch_tiled<256, 256>(A, W, residual, C, f32out, M, N, K, s);
  }
  const int S = plan_tiled_split(M, N, K);
  const size_t need = S > 1 ? (size_t)S * M * N * sizeof(float) : 0;
  TS_REQUIRE(need == 0 || (ws != nullptr && ws_bytes >= need), TS_ERR_WORKSPACE,
             "ts_gemm_bf16: workspace %zu bytes < required %zu", ws_bytes, need);
  return launch_tiled<128, 128>(A, W, residual, C, f32out, M, N, K, s, S, reinterpret_cast<float*>(ws));
}

int launch_moe_gemm(const ts_bf16* A, const int32_t* row_map, int row_div, const ts_bf16* W, const int32_t* offsets,
                    ts_bf16* C, int rows, int E, int N, int K, hipStream_t s) {
  if (rows == 0) return TS_OK;
  SkinnyArgs a{};
  a.A = A; a.row_map = row_map; a.row_div = row_div; a.W = W; a.offsets = offsets; a.residual = nullptr; a.C = C;
  a.partial = nullptr; a.M = rows; a.N = N; a.K = K; a.kslice = (int)round_up((size_t)K, 128); a.S = 1; a.f32out = 0;
  a.w_group_stride = (long)N * K;
  int NT = (cdiv(N, 128) * E >= 448) ? 2 : 1;
  // Row tile: sized for the average expert load; larger experts loop over row blocks.
  const int avg = cdiv(rows, E);
  // (96 rows keep two workgroups per CU and take a 64-row average with its usual spread in one
  // pass: 4.5 TB/s on 8 experts x 64 rows against 3.8 with 128-row tiles and 3.2 with 64-row tiles)
  const int mrows = avg <= 8 ? 16 : (avg <= 20 ? 32 : (avg <= 44 ? 64 : (avg <= 72 ? 96 : 128)));
  int waves = 4;
  if (mrows > 32) {
    // Wider workgroups share one activation slab among more weight rows and keep more loads in flight.  Same
    // load model as the dense plan (workgroups per CU, activation re-reads), with the measured bonus of the
    // seven/eight-wave form at equal width.  8 experts x ~64 rows, H = 4096, F = 14336: gate/up 428 -> 363 us
    // (7 waves x 32 rows), down 211 -> 189 us (8 waves x 16 rows); the other combinations measured worse.
    auto score = [&](int w, int nt) {
      const int cols = 16 * w * nt;
      const long wgs = (long)cdiv(N, cols) * E;
      const double quant = (double)((wgs + 255) / 256 * 256) / (double)wgs;
      return quant * (1.0 + 0.35 * mrows / cols) * (w > 4 ? 0.9 : 1.0);
    };
    double best = score(4, NT);
    const int cand[2][2] = {{7, 2}, {8, 1}};
    for (const auto& c : cand) {
      const double sc = score(c[0], c[1]);
      if (sc < best) {
        best = sc;
        waves = c[0];
        NT = c[1];
      }
    }
  }
  dim3 grid(cdiv(N, 16 * waves * NT), 1, E);
  launch_skinny<true>(a, mrows, NT, grid, s, waves);
  TS_LAUNCH_CHECK("moe_gemm");
  return TS_OK;
}

}  // namespace ts
