// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] * W[N,K]^T with fused epilogues.
//
// Tiling (wave64, v_mfma_f32_32x32x16_bf16):
//   block tile BM x BN with WGM x WGN waves, wave tile (BM/WGM) x (BN/WGN);
//   K is staged through LDS in steps of BK = 64 (double buffered, one barrier per step), with two
//   further K-tiles in flight in registers (prefetch distance 2);
//   global -> registers -> LDS with 16-byte accesses; LDS rows are padded by 16 bytes so that
//   the 16-byte operand reads of 16 consecutive lanes fall into distinct banks.
// Operand roles: the weight rows are the MFMA "A" operand and the token rows the "B" operand,
// i.e. the instruction produces a tile of C^T.  A lane then owns, for one token, quads of
// four consecutive output features, which is what the epilogues want (8-byte bf16 /
// 16-byte fp32 accesses to C, the cache and the residual stream); the tile is re-laid through
// LDS before the epilogue so those accesses are also contiguous across lanes.
// K is walked in order by every tile shape, so an output element is the same fp32 sequence
// regardless of M, of the tile shape and of which rows share the launch.
// Tiles are numbered so that the 8 XCDs (round-robin block dispatch) each work on a
// contiguous range of tiles that share activations in their own L2.
//
// Two main loops share the tile numbering and the epilogue:
//   gemm_dlds_kernel  operands go global -> LDS directly (global_load_lds_dwordx4: a wave writes 64
//                     consecutive 16-byte chunks at a wave-uniform LDS address), no register staging,
//                     no LDS stores; unpadded 128-byte LDS rows with an XOR swizzle of the chunk
//                     position; ring of NS stages with one raw barrier per K-step, loads awaited with
//                     vmcnt(0) by the waves that issued them.  Needs K % 64 == 0.  Tiles 256x128 and 256x256 (half the L2 -> LDS
//                     bytes per FLOP of 128x128).
//   gemm_mfma_kernel  the register-staged loop described above: K tails, small problems.

#include <cmath>

#include "epilogue.h"
#include "gemm.h"

#ifndef SPECA_EBU
#define SPECA_EBU EB
#endif
#ifndef SPECA_SPREAD_LOADS
#define SPECA_SPREAD_LOADS 1
#endif

namespace speca {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;
constexpr int LDS_STRIDE = BK + 8;   // elements; 144-byte rows

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // first-class vector: stays in registers

// XCD-aware tile id: blocks b, b+8, b+16, ... run on the same XCD; give them neighbouring tiles
// (the grid is rounded up to a multiple of 8; surplus blocks leave at once).  Inside an XCD's
// range tiles are walked in groups of group_m M-panels, N fastest across the group's panels,
// so that the tiles in flight at one time form a compact rectangle and share operand panels
// in that XCD's L2.
__device__ __forceinline__ bool tile_coords(int tiles_m, int tiles_n, int group_m, int* tm, int* tn) {
  const int bid = blockIdx.x;
  const int per_xcd = gridDim.x / 8;
  const int tile = (bid % 8) * per_xcd + bid / 8;
  if (tile >= tiles_m * tiles_n) return false;
  const int per_group = group_m * tiles_n;
  const int g = tile / per_group;
  const int first = g * group_m;
  const int h = tiles_m - first < group_m ? tiles_m - first : group_m;
  const int r = tile - g * per_group;
  *tm = first + r % h;
  *tn = r / h;
  return true;
}

// Epilogue of one block tile.  acc[i][j][4*jj + ii] = C[m][n] with m = wm*WM + j*32 + l32,
// n = wn*WN + i*32 + 8*jj + 4*lhi + ii inside the tile.  The tile goes through LDS (fp32, rows padded
// by 16 bytes: conflict-free for the 16-byte writes of 16 consecutive lanes), EH rows at a time, so
// that every global access of the epilogue is a contiguous run along n: a half-wave covers one
// 512-byte (fp32) / 256-byte (bf16) row segment.  Cs must hold EH x (BN + 4) floats; the operand
// buffers it overlays must be dead (all waves past their last read, no load in flight).
template <int BM, int BN, int WGM, int WGN, int MODE, int EH>
__device__ __forceinline__ void tile_epilogue(floatx16 (&acc)[BN / WGN / 32][BM / WGM / 32], float* Cs, int m0, int n0, int M, int N,
                                              const GemmEpi& epi) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int CST = BN + 4;                        // floats per staged row
  constexpr int QPR = BN / 4;                        // quads per row
  constexpr int RPP = NT / QPR;                      // rows per pass
  constexpr int PASSES = EH / RPP;
  static_assert(BM % EH == 0 && EH % WM == 0 && NT % QPR == 0 && EH % RPP == 0, "epilogue shape");
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int qc = (tid % QPR) * 4, qr = tid / QPR;
  const int n = n0 + qc;
  const bool live = n < N;
  float bias[4] = {0.f, 0.f, 0.f, 0.f};
  if (live && epi.bias) Store4<bf16_t>::ld(static_cast<const bf16_t*>(epi.bias) + n, bias);
  // block-uniform row table when the whole tile lies inside one batch row: scalar loads
  const int m_last = (m0 + BM < M ? m0 + BM : M) - 1;
  int i_first = 0;
  bool uniform = false;
  BranchRow<bf16_t> br;
  if (MODE == EPI_BRANCH) {
    i_first = m0 / epi.tokens;
    uniform = i_first == m_last / epi.tokens;
    if (uniform) br = branch_row<bf16_t>(epi, i_first, m0);
  }
#pragma unroll 1
  for (int h = 0; h < BM / EH; ++h) {
    __syncthreads();                                 // operand buffers / previous part consumed
    if (wm * WM / EH == h) {
#pragma unroll
      for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const int r = wm * WM - h * EH + j * 32 + l32, c = wn * WN + i * 32 + 8 * jj + 4 * lhi;
            *reinterpret_cast<float4*>(Cs + r * CST + c) =
                make_float4(acc[i][j][4 * jj], acc[i][j][4 * jj + 1], acc[i][j][4 * jj + 2], acc[i][j][4 * jj + 3]);
          }
    }
    __syncthreads();
    if (!live) continue;
    const int mh = m0 + h * EH;                      // first global row of this part
    if (MODE == EPI_BRANCH) {
      // batches of EB rows: all loads of the batch are issued before its first store
      // (fewer when the accumulators of a later part are still live: 128 registers for a 64x128 wave tile)
      constexpr int EBMAX = (BM / EH > 1) ? 1 : 4;
      constexpr int EB = PASSES % EBMAX == 0 ? EBMAX : (PASSES % 2 == 0 ? 2 : 1);
      if (uniform) {
        constexpr int EBU = SPECA_EBU;
        float g4[4];
        Store4<float>::ld(br.gate + n, g4);
        for (int p0 = 0; p0 < PASSES; p0 += EBU) {
          BranchRegs<bf16_t> regs[EBU];
#pragma unroll
          for (int u = 0; u < EBU; ++u) {
            const int r = qr + (p0 + u) * RPP;
            if (mh + r < M) branch_load_u<bf16_t>(epi, br, h * EH + r, mh + r, n, regs[u]);
          }
#pragma unroll
          for (int u = 0; u < EBU; ++u) {
            const int r = qr + (p0 + u) * RPP;
            if (mh + r < M) {
              const float4 t = *reinterpret_cast<const float4*>(Cs + r * CST + qc);
              const float v[4] = {t.x + bias[0], t.y + bias[1], t.z + bias[2], t.w + bias[3]};
              branch_finish_u<bf16_t>(epi, br, h * EH + r, mh + r, n, v, g4, regs[u]);
            }
          }
        }
      } else {
        for (int p0 = 0; p0 < PASSES; p0 += EB) {
          BranchRegs<bf16_t> regs[EB];
#pragma unroll
          for (int u = 0; u < EB; ++u) {
            const int m = mh + qr + (p0 + u) * RPP;
            if (m < M) branch_load<bf16_t>(epi, m, n, regs[u]);
          }
#pragma unroll
          for (int u = 0; u < EB; ++u) {
            const int r = qr + (p0 + u) * RPP;
            const int m = mh + r;
            if (m < M) {
              const float4 t = *reinterpret_cast<const float4*>(Cs + r * CST + qc);
              const float v[4] = {t.x + bias[0], t.y + bias[1], t.z + bias[2], t.w + bias[3]};
              branch_finish<bf16_t>(epi, m, n, v, regs[u]);
            }
          }
        }
      }
    } else {
#pragma unroll 4
      for (int r = qr; r < EH; r += RPP) {
        const int m = mh + r;
        if (m < M) {
          const float4 t = *reinterpret_cast<const float4*>(Cs + r * CST + qc);
          float v[4] = {t.x + bias[0], t.y + bias[1], t.z + bias[2], t.w + bias[3]};
          epilogue_apply<bf16_t, MODE>(epi, m, n, v);
        }
      }
    }
  }
}

// KTAIL: K is not a multiple of BK; the last operand tile is zero-filled by predicated loads.
// SF ("store first"): the LDS stores of the next tile are issued ahead of the MFMAs of the current
// one instead of behind them.  Measured: faster for long K loops on large outputs (K >= 2048:
// +5..11 %), slower for short ones (K = 1152), so the host picks by shape.
template <int BM, int BN, int WGM, int WGN, int MODE, bool KTAIL, bool SF>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_mfma_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                                   const uint16_t* __restrict__ W, int64_t ldw, int M, int N, int K,
                                                                   int tiles_m, int tiles_n, int group_m, GemmEpi epi) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;      // wave tile
  constexpr int TM = WM / 32, TN = WN / 32;        // MFMA tiles per wave
  constexpr int A_CHUNKS = BM * (BK / 8) / NT;     // 16-byte chunks per thread per stage
  constexpr int W_CHUNKS = BN * (BK / 8) / NT;
  static_assert(BM * (BK / 8) % NT == 0 && BN * (BK / 8) % NT == 0, "tile does not divide among the threads");
  extern __shared__ __align__(16) uint16_t smem[];
  uint16_t* As = smem;                              // [2][BM][LDS_STRIDE]
  uint16_t* Ws = smem + 2 * BM * LDS_STRIDE;        // [2][BN][LDS_STRIDE]

  int tm, tn;
  if (!tile_coords(tiles_m, tiles_n, group_m, &tm, &tn)) return;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int l32 = lane & 31, lhi = lane >> 5;

  floatx16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

  // Operand staging: two register sets, i.e. two K-tiles in flight per block (prefetch distance 2)
  // on top of the LDS double buffer.  Loads are branch-free: rows beyond M / N are clamped to the
  // last row (their results are never stored) and tiles beyond K re-read the last tile, so the
  // compiler can count outstanding loads exactly instead of draining them at every branch.
  const int nk = (K + BK - 1) / BK;
  const uint16_t* pa[A_CHUNKS];
  const uint16_t* pw[W_CHUNKS];
  int kca[A_CHUNKS], kcw[W_CHUNKS];
#pragma unroll
  for (int c = 0; c < A_CHUNKS; ++c) {
    const int id = tid + c * NT;
    const int row = id >> 3;
    kca[c] = (id & 7) * 8;
    const int m = m0 + row < M ? m0 + row : M - 1;
    pa[c] = A + static_cast<int64_t>(m) * lda + kca[c];
  }
#pragma unroll
  for (int c = 0; c < W_CHUNKS; ++c) {
    const int id = tid + c * NT;
    const int row = id >> 3;
    kcw[c] = (id & 7) * 8;
    const int n = n0 + row < N ? n0 + row : N - 1;
    pw[c] = W + static_cast<int64_t>(n) * ldw + kcw[c];
  }
  u32x4 ra0[A_CHUNKS], rw0[W_CHUNKS], ra1[A_CHUNKS], rw1[W_CHUNKS];
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

#define SPECA_LOADG(ra, rw, kt_)                                                                               \
  {                                                                                                            \
    const int k0_ = ((kt_) < nk ? (kt_) : nk - 1) * BK;                                                        \
    _Pragma("unroll") for (int c = 0; c < A_CHUNKS; ++c) {                                                     \
      if (KTAIL) ra[c] = (k0_ + kca[c] < K) ? *reinterpret_cast<const u32x4*>(pa[c] + k0_) : zero4;            \
      else ra[c] = *reinterpret_cast<const u32x4*>(pa[c] + k0_);                                               \
    }                                                                                                          \
    _Pragma("unroll") for (int c = 0; c < W_CHUNKS; ++c) {                                                     \
      if (KTAIL) rw[c] = (k0_ + kcw[c] < K) ? *reinterpret_cast<const u32x4*>(pw[c] + k0_) : zero4;            \
      else rw[c] = *reinterpret_cast<const u32x4*>(pw[c] + k0_);                                               \
    }                                                                                                          \
  }
#define SPECA_STOREL(ra, rw, buf)                                                                              \
  {                                                                                                            \
    _Pragma("unroll") for (int c = 0; c < A_CHUNKS; ++c) {                                                     \
      const int id = tid + c * NT;                                                                             \
      *reinterpret_cast<u32x4*>(As + ((buf) * BM + (id >> 3)) * LDS_STRIDE + (id & 7) * 8) = ra[c];            \
    }                                                                                                          \
    _Pragma("unroll") for (int c = 0; c < W_CHUNKS; ++c) {                                                     \
      const int id = tid + c * NT;                                                                             \
      *reinterpret_cast<u32x4*>(Ws + ((buf) * BN + (id >> 3)) * LDS_STRIDE + (id & 7) * 8) = rw[c];            \
    }                                                                                                          \
  }
#define SPECA_COMPUTE(buf)                                                                                     \
  {                                                                                                            \
    const uint16_t* as = As + ((buf) * BM + wm * WM + l32) * LDS_STRIDE + lhi * 8;                             \
    const uint16_t* ws = Ws + ((buf) * BN + wn * WN + l32) * LDS_STRIDE + lhi * 8;                             \
    _Pragma("unroll") for (int ks = 0; ks < BK / 16; ++ks) {                                                   \
      bf16x8 fa[TM], fw[TN];                                                                                   \
      _Pragma("unroll") for (int j = 0; j < TM; ++j) fa[j] = *reinterpret_cast<const bf16x8*>(as + j * 32 * LDS_STRIDE + ks * 16); \
      _Pragma("unroll") for (int i = 0; i < TN; ++i) fw[i] = *reinterpret_cast<const bf16x8*>(ws + i * 32 * LDS_STRIDE + ks * 16); \
      _Pragma("unroll") for (int i = 0; i < TN; ++i) _Pragma("unroll") for (int j = 0; j < TM; ++j)            \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);                  \
    }                                                                                                          \
  }

  SPECA_LOADG(ra0, rw0, 0);
  SPECA_LOADG(ra1, rw1, 1);
  SPECA_STOREL(ra0, rw0, 0);
  SPECA_LOADG(ra0, rw0, 2);
  __syncthreads();
  if (SF) {
    for (int kt = 0; kt < nk; kt += 2) {
      SPECA_STOREL(ra1, rw1, 1);             // tile kt+1 -> buffer 1 (last read before the previous barrier)
      SPECA_LOADG(ra1, rw1, kt + 3);
      SPECA_COMPUTE(0);                      // tile kt
      __syncthreads();
      SPECA_STOREL(ra0, rw0, 0);             // tile kt+2 -> buffer 0
      SPECA_LOADG(ra0, rw0, kt + 4);
      if (kt + 1 < nk) SPECA_COMPUTE(1);     // tile kt+1
      __syncthreads();
    }
  } else {
    for (int kt = 0; kt < nk; kt += 2) {
      SPECA_COMPUTE(0);                      // tile kt
      SPECA_STOREL(ra1, rw1, 1);             // tile kt+1 -> buffer 1
      SPECA_LOADG(ra1, rw1, kt + 3);
      __syncthreads();
      if (kt + 1 < nk) SPECA_COMPUTE(1);     // tile kt+1
      SPECA_STOREL(ra0, rw0, 0);             // tile kt+2 -> buffer 0
      SPECA_LOADG(ra0, rw0, kt + 4);
      __syncthreads();
    }
  }
#undef SPECA_LOADG
#undef SPECA_STOREL
#undef SPECA_COMPUTE

  tile_epilogue<BM, BN, WGM, WGN, MODE, BM>(acc, reinterpret_cast<float*>(smem), m0, n0, M, N, epi);
}

// ---------------------------------------------------------------------------------------------
// Direct-to-LDS main loop.
//
// LDS stage = [BM + BN rows][64 bf16], rows unpadded (128 bytes = 8 chunks of 16 bytes).  Chunk c of
// row r sits at chunk position c ^ swz(r), swz(r) = (r & 7) ^ ((r >> 3) & 1): the 16 lanes that read
// the same chunk index of 16 consecutive rows then touch all 64 banks exactly once.
// Loader: one load instruction fills 8 rows (64 chunks, 1 KiB, contiguous in LDS); lane l supplies
// the chunk stored at position l % 8 of row l / 8, i.e. source chunk (l % 8) ^ swz(row), and the
// hardware places lane l's 16 bytes at the wave-uniform LDS address + 16 l.  A loader wave owns the
// row groups wl, wl + NL, ... (NL loader waves, NL even, so swz depends only on the lane and the
// parity of wl).  Rows beyond M / N are clamped to the last row (never stored).
//
// Completion of these loads is only ever awaited with vmcnt(0).  A partial wait ("all but the newest
// six have landed") assumes they complete in issue order; they do not reliably: a 3-stage ring built
// on vmcnt(6) passed every isolated test and then delivered stale operand rows (32-row groups, a few
// launches per step) once four row groups ran side by side.  Two loads-in-flight stages with
// vmcnt(0)-only waits are obtained by splitting the waves into two loader groups instead: group g
// loads the K-steps of parity g, so at its wait a group has exactly one step outstanding (the one
// everybody needs next) while the other group's step stays in flight.
// Ring discipline per K-step kt (NS = 2: every wave loads every step; NS = 3: two groups):
//   the step's loader waves wait vmcnt(0); barrier (the step is in LDS, everyone is done reading the
//   previous step's stage); the same waves issue step kt + NS - 1 into the stage just freed; compute.
#define SPECA_GLL(src, dst)                                                                                       \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),                         \
                                   (__attribute__((address_space(3))) void*)(dst), 16, 0, 0)

// Rows of the tile staged through LDS per epilogue part: the whole tile when it fits into the ring's
// LDS, else half of it (no LDS beyond the ring: 128x128 stays at 64 KiB, two blocks per CU with room).
constexpr int dlds_epilogue_rows(int BM, int BN, int NS) {
  return BM * (BN + 4) * 4 <= NS * (BM + BN) * BK * 2 ? BM : BM / 2;
}

template <int BM, int BN, int WGM, int WGN, int NS, int MODE>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_dlds_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                                   const uint16_t* __restrict__ W, int64_t ldw, int M, int N, int K,
                                                                   int tiles_m, int tiles_n, int group_m, GemmEpi epi) {
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(NS == 2 || NS == 3, "ring depth");
  constexpr int NL = NS == 3 ? NW / 2 : NW;                  // loader waves per K-step
  constexpr int AG = BM / 8 / NL, WG = BN / 8 / NL;          // 8-row groups (one load instruction each) per loader wave
  static_assert(BM / 8 % NL == 0 && BN / 8 % NL == 0 && NL % 2 == 0, "row groups must divide among an even number of loader waves");
  constexpr int STAGE = (BM + BN) * BK;                      // elements per stage
  constexpr int EH = dlds_epilogue_rows(BM, BN, NS);
  extern __shared__ __align__(16) uint16_t smem[];

  int tm, tn;
  if (!tile_coords(tiles_m, tiles_n, group_m, &tm, &tn)) return;
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int l32 = lane & 31, lhi = lane >> 5;

  floatx16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

  const int nk = K / BK;
  const int grp = wave / NL, wl = wave % NL;                 // loader group (NS = 3) and index inside it
  const int lrow = lane >> 3;
  const int lchunk = (lane & 7) ^ lrow ^ (wl & 1);
  const uint16_t* pa[AG];
  const uint16_t* pw[WG];
#pragma unroll
  for (int g = 0; g < AG; ++g) {
    const int row = (wl + g * NL) * 8 + lrow;
    const int m = m0 + row < M ? m0 + row : M - 1;
    pa[g] = A + static_cast<int64_t>(m) * lda + lchunk * 8;
  }
#pragma unroll
  for (int g = 0; g < WG; ++g) {
    const int row = (wl + g * NL) * 8 + lrow;
    const int n = n0 + row < N ? n0 + row : N - 1;
    pw[g] = W + static_cast<int64_t>(n) * ldw + lchunk * 8;
  }
  // reader: row = base + l32 (bases are multiples of 32), chunk 2 ks + lhi
  const int sw = (l32 & 7) ^ ((l32 >> 3) & 1);
  int coff[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) coff[ks] = ((2 * ks + lhi) ^ sw) * 8;

#define SPECA_LOADS(st, kt_)                                                                                      \
  {                                                                                                               \
    const int k0_ = (kt_) * BK;                                                                                   \
    _Pragma("unroll") for (int g = 0; g < AG; ++g) SPECA_GLL(pa[g] + k0_, smem + (st) * STAGE + (wl + g * NL) * 512);           \
    _Pragma("unroll") for (int g = 0; g < WG; ++g) SPECA_GLL(pw[g] + k0_, smem + (st) * STAGE + BM * BK + (wl + g * NL) * 512); \
  }
#define SPECA_LDFRAG(fa_, fw_, ks_)                                                                               \
  {                                                                                                               \
    _Pragma("unroll") for (int j = 0; j < TM; ++j) fa_[j] = *reinterpret_cast<const bf16x8*>(as + j * 32 * BK + coff[ks_]); \
    _Pragma("unroll") for (int i = 0; i < TN; ++i) fw_[i] = *reinterpret_cast<const bf16x8*>(ws + i * 32 * BK + coff[ks_]); \
  }
#define SPECA_MFMAS(fa_, fw_)                                                                                     \
  {                                                                                                               \
    _Pragma("unroll") for (int i = 0; i < TN; ++i) _Pragma("unroll") for (int j = 0; j < TM; ++j)                 \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw_[i], fa_[j], acc[i][j], 0, 0, 0);                    \
  }
  // fragments of the next 16-wide K slice are requested before the MFMAs of the current one
#define SPECA_COMPUTE(st)                                                                                         \
  {                                                                                                               \
    const uint16_t* as = smem + (st) * STAGE + (wm * WM + l32) * BK;                                              \
    const uint16_t* ws = smem + (st) * STAGE + BM * BK + (wn * WN + l32) * BK;                                    \
    bf16x8 fa0[TM], fw0[TN], fa1[TM], fw1[TN];                                                                    \
    SPECA_LDFRAG(fa0, fw0, 0);                                                                                    \
    SPECA_LDFRAG(fa1, fw1, 1);                                                                                    \
    SPECA_MFMAS(fa0, fw0);                                                                                        \
    SPECA_LDFRAG(fa0, fw0, 2);                                                                                    \
    SPECA_MFMAS(fa1, fw1);                                                                                        \
    SPECA_LDFRAG(fa1, fw1, 3);                                                                                    \
    SPECA_MFMAS(fa0, fw0);                                                                                        \
    SPECA_MFMAS(fa1, fw1);                                                                                        \
    /* keep that order in the instruction stream: two slices of fragments in flight ahead of the MFMAs */         \
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * (TM + TN), 0);                                                \
    __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);                                                      \
    __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);                                                      \
    __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);                                                      \
    __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);                                                      \
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * TM * TN, 0);                                                  \
  }
  // The same compute with the loads of a later K-step spread between its MFMAs.  Issued in a burst right
  // after the barrier, the loads (a few address instructions each) hold every wave's in-order issue while the
  // matrix cores idle; here loads and MFMAs sit in one scheduling region (no branch: past the last K-step the
  // last tile is re-read into the free stage, never consumed, awaited before the epilogue) and the group
  // barriers ask for the loads one at a time between MFMAs.
  constexpr int LPW = AG + WG;                               // loads per loader wave and step
  // Only with the 3-stage ring: there a load has two K-steps to land; with two stages (one step of lead) issuing
  // the loads later in the step cost more at the next wait than the burst did (measured -3..-5 %).
  constexpr bool SPREAD = NS == 3 && LPW % 4 == 0 && ((TM * TN) % (LPW / 4) == 0 || LPW / 4 == 3) && SPECA_SPREAD_LOADS;
#ifndef SPECA_ONE_AHEAD
#define SPECA_ONE_AHEAD 1
#endif
#ifndef SPECA_FINE_READS
#define SPECA_FINE_READS 1
#endif
#ifndef SPECA_EARLY_LOADS
#define SPECA_EARLY_LOADS 1
#endif
  // Two stages (one K-step of lead): the loads go one per MFMA from the start of the step, so they are all out
  // within its first slice or two instead of holding the issue of every wave up front (+6..8 % on the 256x256 tile).
  constexpr bool EARLY = NS == 2 && LPW <= 2 * TM * TN && SPECA_EARLY_LOADS;
#define SPECA_SLICE_GROUPS                                                                                        \
  {                                                                                                               \
    constexpr int LPS_ = LPW / 4, MM_ = TM * TN;                                                                  \
    if (MM_ % LPS_ == 0) {                                                                                        \
      _Pragma("unroll") for (int l = 0; l < LPS_; ++l) {                                                          \
        __builtin_amdgcn_sched_group_barrier(0x008, MM_ / LPS_, 0);                                               \
        __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);                                                        \
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                                        \
      }                                                                                                           \
    } else { /* 4 MFMAs, 3 loads */                                                                               \
      _Pragma("unroll") for (int l = 0; l < 3; ++l) {                                                             \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                        \
        __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);                                                        \
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                                        \
      }                                                                                                           \
      __builtin_amdgcn_sched_group_barrier(0x008, MM_ - 3, 0);                                                    \
    }                                                                                                             \
  }
#define SPECA_COMPUTE_L(st, new_, ktl_)                                                                           \
  {                                                                                                               \
    const uint16_t* as = smem + (st) * STAGE + (wm * WM + l32) * BK;                                              \
    const uint16_t* ws = smem + (st) * STAGE + BM * BK + (wn * WN + l32) * BK;                                    \
    bf16x8 fa0[TM], fw0[TN], fa1[TM], fw1[TN];                                                                    \
    SPECA_LDFRAG(fa0, fw0, 0);                                                                                    \
    SPECA_LDFRAG(fa1, fw1, 1);                                                                                    \
    SPECA_LOADS(new_, (ktl_) < nk ? (ktl_) : nk - 1);                                                             \
    SPECA_MFMAS(fa0, fw0);                                                                                        \
    SPECA_LDFRAG(fa0, fw0, 2);                                                                                    \
    SPECA_MFMAS(fa1, fw1);                                                                                        \
    SPECA_LDFRAG(fa1, fw1, 3);                                                                                    \
    SPECA_MFMAS(fa0, fw0);                                                                                        \
    SPECA_MFMAS(fa1, fw1);                                                                                        \
    if (EARLY && SPECA_ONE_AHEAD && LPW <= TM * TN && TM + TN <= TM * TN) {                                       \
      /* one slice of fragments ahead is enough when its reads go out one per MFMA of the current slice */        \
      __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);                                                    \
      _Pragma("unroll") for (int l = 0; l < TM * TN; ++l) {                                                       \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                        \
        if (l < LPW) { __builtin_amdgcn_sched_group_barrier(0x002, 4, 0); __builtin_amdgcn_sched_group_barrier(0x020, 1, 0); } \
        if (l < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                       \
      }                                                                                                           \
      _Pragma("unroll") for (int q = 0; q < 2; ++q)                                                               \
        _Pragma("unroll") for (int l = 0; l < TM * TN; ++l) {                                                     \
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                      \
          if (l < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                     \
        }                                                                                                         \
      __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);                                                    \
    } else {                                                                                                      \
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * (TM + TN), 0);                                                \
    if (EARLY) {                                                                                                  \
      constexpr int L0_ = LPW < TM * TN ? LPW : TM * TN, L1_ = LPW - L0_;   /* loads placed in slices 0 and 1 */     \
      _Pragma("unroll") for (int l = 0; l < L0_; ++l) {                                                           \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                        \
        __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);                                                        \
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                                        \
      }                                                                                                           \
      if (TM * TN - L0_ > 0) __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - L0_, 0);                       \
      if (SPECA_FINE_READS && L1_ == 0 && TM + TN <= TM * TN) {                                                   \
        /* the next slice's fragment reads go one per MFMA too */                                                 \
        _Pragma("unroll") for (int q = 0; q < 2; ++q) {                                                           \
          _Pragma("unroll") for (int l = 0; l < TM + TN; ++l) {                                                   \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                    \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                    \
          }                                                                                                       \
          if (TM * TN - (TM + TN) > 0) __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - (TM + TN), 0);       \
        }                                                                                                         \
        __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);                                                  \
      } else {                                                                                                    \
      __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);                                                    \
      _Pragma("unroll") for (int l = 0; l < L1_; ++l) {                                                           \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                        \
        __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);                                                        \
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                                        \
      }                                                                                                           \
      if (TM * TN - L1_ > 0) __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - L1_, 0);                       \
      __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);                                                    \
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * TM * TN, 0);                                                \
      }                                                                                                           \
    } else {                                                                                                      \
    SPECA_SLICE_GROUPS;                                                                                           \
    if (SPECA_FINE_READS && LPW / 4 == 3 && TM * TN == 4 && TM + TN == 4) {                                       \
      /* slices 1 and 2: the fragment reads of the slice after next go one per MFMA as well */                    \
      _Pragma("unroll") for (int q = 0; q < 2; ++q) {                                                             \
        _Pragma("unroll") for (int l = 0; l < 3; ++l) {                                                           \
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                      \
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                      \
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);                                                      \
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                                      \
        }                                                                                                         \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                        \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                        \
      }                                                                                                           \
      SPECA_SLICE_GROUPS;                                                                                         \
    } else {                                                                                                      \
    __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);                                                      \
    SPECA_SLICE_GROUPS;                                                                                           \
    __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);                                                      \
    SPECA_SLICE_GROUPS;                                                                                           \
    SPECA_SLICE_GROUPS;                                                                                           \
    }                                                                                                             \
    }                                                                                                             \
    }                                                                                                             \
  }
  constexpr int WAIT_VM0 = 0x0F70;                           // s_waitcnt vmcnt(0), other counters untouched
  // prologue: steps 0 .. NS-2, each by its loader waves
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < nk && (NS == 2 || grp == (s & 1))) SPECA_LOADS(s, s);
  // One K-step with compile-time stage numbers and loader parity (the ring has period NS, the loader
  // groups period 2: the loop body is unrolled over their common period so every LDS address is an
  // immediate offset).
#define SPECA_STEP(kt_, cur_, new_, par_)                                                                         \
  {                                                                                                               \
    const bool mine_ = NS == 2 || grp == (par_);             /* wave-uniform */                                    \
    if (mine_) __builtin_amdgcn_s_waitcnt(WAIT_VM0);         /* my only outstanding loads are those of this step */ \
    __builtin_amdgcn_s_barrier();                                                                                 \
    if (SPREAD || EARLY) {                                                                                        \
      if (mine_) SPECA_COMPUTE_L(cur_, new_, (kt_) + NS - 1)                                                      \
      else SPECA_COMPUTE(cur_)                                                                                    \
    } else {                                                                                                      \
      if (mine_ && (kt_) + NS - 1 < nk) SPECA_LOADS(new_, (kt_) + NS - 1);                                        \
      SPECA_COMPUTE(cur_);                                                                                        \
    }                                                                                                             \
  }
  if (NS == 2) {
    for (int kt = 0; kt < nk; kt += 2) {
      SPECA_STEP(kt, 0, 1, 0);
      if (kt + 1 < nk) SPECA_STEP(kt + 1, 1, 0, 0);
    }
  } else {
    for (int kt = 0; kt < nk; kt += 6) {
      SPECA_STEP(kt, 0, 2, 0);
      if (kt + 1 < nk) SPECA_STEP(kt + 1, 1, 0, 1);
      if (kt + 2 < nk) SPECA_STEP(kt + 2, 2, 1, 0);
      if (kt + 3 < nk) SPECA_STEP(kt + 3, 0, 2, 1);
      if (kt + 4 < nk) SPECA_STEP(kt + 4, 1, 0, 0);
      if (kt + 5 < nk) SPECA_STEP(kt + 5, 2, 1, 1);
    }
  }
#undef SPECA_STEP
  __builtin_amdgcn_s_waitcnt(WAIT_VM0);                      // nothing is outstanding here; kept as a guard before LDS is reused
#undef SPECA_COMPUTE
#undef SPECA_COMPUTE_L
#undef SPECA_SLICE_GROUPS
#undef SPECA_MFMAS
#undef SPECA_LDFRAG
#undef SPECA_LOADS

  tile_epilogue<BM, BN, WGM, WGN, MODE, EH>(acc, reinterpret_cast<float*>(smem), m0, n0, M, N, epi);
}

template <int BM, int BN, int WGM, int WGN, int NS>
Error launch_dlds(const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi, hipStream_t st) {
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const int64_t nblk = static_cast<int64_t>(tiles_m) * tiles_n;
  if (nblk > 0x7FFFFFF0) SPECA_FAIL(SPECA_EINVAL, "gemm: too many tiles");
  if (K % BK != 0 || K < BK) SPECA_FAIL(SPECA_EINVAL, "gemm: direct-to-LDS loop needs K %% 64 == 0");
  constexpr int EH = dlds_epilogue_rows(BM, BN, NS);
  const size_t smem_ops = static_cast<size_t>(NS) * (BM + BN) * BK * sizeof(uint16_t);
  const size_t smem_epi = static_cast<size_t>(EH) * (BN + 4) * sizeof(float);
  const size_t smem = smem_ops > smem_epi ? smem_ops : smem_epi;
  const uint16_t* a = static_cast<const uint16_t*>(A);
  const uint16_t* w = static_cast<const uint16_t*>(W);
  dim3 grid(static_cast<unsigned>((nblk + 7) / 8 * 8));
  const int group_m = tiles_m < 4 ? tiles_m : 4;
#define SPECA_LAUNCH(MODE_)                                                                                       \
  {                                                                                                               \
    auto kern = gemm_dlds_kernel<BM, BN, WGM, WGN, NS, MODE_>;                                                    \
    static bool attr_set = false;   /* more than 64 KB of dynamic LDS must be requested once per kernel */          \
    if (smem > 64 * 1024 && !attr_set) {                                                                          \
      SPECA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem))); \
      attr_set = true;                                                                                            \
    }                                                                                                             \
    kern<<<grid, WGM * WGN * 64, smem, st>>>(a, lda, w, ldw, M, N, K, tiles_m, tiles_n, group_m, epi);             \
  }
  switch (epi.mode) {
    case EPI_STORE: SPECA_LAUNCH(EPI_STORE) break;
    case EPI_GELU: SPECA_LAUNCH(EPI_GELU) break;
    case EPI_SILU: SPECA_LAUNCH(EPI_SILU) break;
    case EPI_F32: SPECA_LAUNCH(EPI_F32) break;
    case EPI_BRANCH: SPECA_LAUNCH(EPI_BRANCH) break;
    default: SPECA_FAIL(SPECA_EINVAL, "gemm: epilogue mode %d", epi.mode);
  }
#undef SPECA_LAUNCH
  SPECA_HIP(hipGetLastError());
  return ok();
}

template <int BM, int BN, int WGM, int WGN>
Error launch_tile(const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi, hipStream_t st) {
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const int64_t nblk = static_cast<int64_t>(tiles_m) * tiles_n;
  if (nblk > 0x7FFFFFF0) SPECA_FAIL(SPECA_EINVAL, "gemm: too many tiles");
  const size_t smem_ops = static_cast<size_t>(2) * (BM + BN) * LDS_STRIDE * sizeof(uint16_t);
  const size_t smem_epi = static_cast<size_t>(BM) * (BN + 4) * sizeof(float);
  const size_t smem = smem_ops > smem_epi ? smem_ops : smem_epi;
  const uint16_t* a = static_cast<const uint16_t*>(A);
  const uint16_t* w = static_cast<const uint16_t*>(W);
  dim3 grid(static_cast<unsigned>((nblk + 7) / 8 * 8));
  const int group_m = tiles_m < 4 ? tiles_m : 4;
  const bool ktail = K % BK != 0;
  const bool store_first = K >= 2048 && static_cast<int64_t>(M) * N >= (int64_t{8} << 20);
#define SPECA_LAUNCH2(MODE_, KT_, SF_)                                                                          \
  {                                                                                                              \
    auto kern = gemm_mfma_kernel<BM, BN, WGM, WGN, MODE_, KT_, SF_>;                                                 \
    static bool attr_set = false;   /* more than 64 KB of dynamic LDS must be requested once per kernel */         \
    if (smem > 64 * 1024 && !attr_set) {                                                                         \
      SPECA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem))); \
      attr_set = true;                                                                                           \
    }                                                                                                            \
    kern<<<grid, WGM * WGN * 64, smem, st>>>(a, lda, w, ldw, M, N, K, tiles_m, tiles_n, group_m, epi);            \
  }
#define SPECA_LAUNCH(MODE_)                       \
  {                                               \
    if (ktail) SPECA_LAUNCH2(MODE_, true, false)  \
    else if (store_first) SPECA_LAUNCH2(MODE_, false, true) \
    else SPECA_LAUNCH2(MODE_, false, false)       \
  }
  switch (epi.mode) {
    case EPI_STORE: SPECA_LAUNCH(EPI_STORE) break;
    case EPI_GELU: SPECA_LAUNCH(EPI_GELU) break;
    case EPI_SILU: SPECA_LAUNCH(EPI_SILU) break;
    case EPI_F32: SPECA_LAUNCH(EPI_F32) break;
    case EPI_BRANCH: SPECA_LAUNCH(EPI_BRANCH) break;
    default: SPECA_FAIL(SPECA_EINVAL, "gemm: epilogue mode %d", epi.mode);
  }
#undef SPECA_LAUNCH
#undef SPECA_LAUNCH2
  SPECA_HIP(hipGetLastError());
  return ok();
}

}  // namespace

bool gemm_mfma_supported(const void* A, int64_t lda, const void* W, int64_t ldw, int N, int K) {
  return (K % 8 == 0) && (lda % 8 == 0) && (ldw % 8 == 0) && (N % 8 == 0) && (reinterpret_cast<uintptr_t>(A) % 16 == 0) &&
         (reinterpret_cast<uintptr_t>(W) % 16 == 0);
}

// ---- tile choice -------------------------------------------------------------------------------------------
// Six kernels can run a given problem; which is fastest depends on how the tile count falls on the chip's compute
// units more than on anything else (a 270-tile launch of one-block-per-CU tiles takes two rounds, a 252-tile one
// takes one), and the row count M varies from call to call: per-sample rejection sends any number of guidance pairs
// to the full pass and the lanes split a batch into row groups.  So the choice is made by a small cost model instead
// of thresholds fitted to particular shapes:
//     time(kernel) = (a + b * ceil(K / 64)) * depth,     depth = ceil(tiles / compute units),
// where kernels whose LDS footprint lets a second block share a compute unit pay 0.65 of a round for every round
// after the first.  a (launch, prologue, epilogue) and b (one 64-wide K-step) were measured in microseconds per
// kernel on the block GEMMs of the DiT-XL/2 shape at M = 256 .. 4096 and on FLUX-sized problems with cold weights;
// over those 45 problems the model's pick is within 2 % of the best kernel everywhere (the thresholds it replaces
// lost 17-26 % at M = 1024, 2048, 2560 and 3072-3584).  Absolute times are off by up to 25 % on long-K problems,
// where every kernel slows down alike; only the ranking is used.
struct TileKind {
  int bm, bn;
  float a, b;          // microseconds
  bool shares_cu;      // a second block fits beside the first
  bool dlds;           // direct-to-LDS loop: K % 64 == 0, M >= 256
  bool wide;           // 256-row tiles: M >= 256
};
constexpr TileKind kTileKinds[6] = {
    {256, 256, 8.0f, 1.115f, false, true, true},    // 0: direct-to-LDS, 2 stages
    {256, 128, 4.1f, 0.844f, false, true, true},    // 1: direct-to-LDS, 2 stages
    {256, 128, 5.4f, 0.710f, false, true, true},    // 2: direct-to-LDS, 3 stages
    {256, 128, 5.6f, 0.810f, false, false, true},   // 3: register-staged
    {128, 128, 5.3f, 0.574f, true, false, false},   // 4: register-staged, two blocks per compute unit
    {128, 64, 4.2f, 0.400f, true, false, false},    // 5: register-staged
};

static int compute_units() {
  static const int n = [] {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu < 1) {
      (void)hipGetLastError();
      cu = 256;
    }
    return cu;
  }();
  return n;
}

static double tile_cost(const TileKind& t, int M, int N, int K) {
  const double tiles = static_cast<double>((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
  const double depth = std::ceil(tiles / compute_units());
  const double one = t.a + t.b * ((K + BK - 1) / BK);
  return t.shares_cu ? one * (1.0 + 0.65 * (depth - 1.0)) : one * depth;
}

// cheapest eligible kernel for the problem; *cost receives its modelled time
static int pick_tile(int M, int N, int K, double* cost) {
  int best = -1;
  double bc = 0.0;
  for (int k = 0; k < 6; ++k) {
    const TileKind& t = kTileKinds[k];
    if (t.dlds && (K % BK != 0 || K < BK)) continue;
    if (t.wide && M < 256) continue;
    const double c = tile_cost(t, M, N, K);
    if (best < 0 || c < bc) { best = k; bc = c; }
  }
  *cost = bc;
  return best;
}

static Error launch_kind(int kind, const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi, hipStream_t st) {
  switch (kind) {
    case 0: return launch_dlds<256, 256, 4, 2, 2>(A, lda, W, ldw, M, N, K, epi, st);
    case 1: return launch_dlds<256, 128, 4, 2, 2>(A, lda, W, ldw, M, N, K, epi, st);
    case 2: return launch_dlds<256, 128, 4, 2, 3>(A, lda, W, ldw, M, N, K, epi, st);
    case 3: return launch_tile<256, 128, 4, 2>(A, lda, W, ldw, M, N, K, epi, st);
    case 4: return launch_tile<128, 128, 2, 2>(A, lda, W, ldw, M, N, K, epi, st);
    default: return launch_tile<128, 64, 2, 2>(A, lda, W, ldw, M, N, K, epi, st);
  }
}

// Row groups of one step that run side by side on their own streams (GemmEpi::shared_chip) share the compute units with
// each other's kernels, which the model above does not price: planned for a quarter of the chip each, four lanes took
// the large tiles of the whole batch and a step got 5 % slower.  What measured best there are the kernels that leave
// room beside them: the 2-stage 256x128 ring (96 KiB of LDS, a 128x64 block of another lane still fits on the compute
// unit), 128x64 tiles for the small N = 1152 GEMM, and the 3-stage ring only for a long-K GEMM of few tiles.
static Error launch_shared(const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi, hipStream_t st) {
  const int64_t t128 = static_cast<int64_t>((M + 127) / 128) * ((N + 127) / 128);
  const int64_t t256 = static_cast<int64_t>((M + 255) / 256) * ((N + 127) / 128);
  if (K % BK == 0 && K >= BK && M >= 256) {
    if (K >= 2048 && t256 >= 32 && t256 < 100) return launch_dlds<256, 128, 4, 2, 3>(A, lda, W, ldw, M, N, K, epi, st);
    if (t256 >= 100 && t256 < 256) return launch_dlds<256, 128, 4, 2, 2>(A, lda, W, ldw, M, N, K, epi, st);
  }
  double cost = 0.0;
  if (t256 >= 256) return launch_kind(pick_tile(M, N, K, &cost), A, lda, W, ldw, M, N, K, epi, st);
  if (t128 >= 200) return launch_tile<128, 128, 2, 2>(A, lda, W, ldw, M, N, K, epi, st);
  return launch_tile<128, 64, 2, 2>(A, lda, W, ldw, M, N, K, epi, st);
}

Error launch_gemm_mfma(const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi, hipStream_t st) {
  if (epi.shared_chip > 1) return launch_shared(A, lda, W, ldw, M, N, K, epi, st);
  double whole = 0.0;
  const int kind = pick_tile(M, N, K, &whole);
  // A little more than one round of 256x256 tiles (the 4096 x 4608 x 1152 fc1 GEMM: 288): the columns that make exactly one
  // round go on the large tile, the remaining columns in a second launch (47 + 13 us against 61 us for the best single
  // kernel).  Column ranges only shift pointers, so this is limited to the epilogues that store into `out`.
  if (epi.mode != EPI_BRANCH && K % BK == 0 && K >= BK && M >= 256) {
    const int tiles_m = (M + 255) / 256;
    const int n1 = (compute_units() / tiles_m) * 256;
    if (n1 >= 256 && n1 < N) {
      double rest = 0.0;
      (void)pick_tile(M, N - n1, K, &rest);
      if (tile_cost(kTileKinds[0], M, n1, K) + rest < 0.9 * whole) {
        SPECA_TRY((launch_dlds<256, 256, 4, 2, 2>(A, lda, W, ldw, M, n1, K, epi, st)));
        GemmEpi tail = epi;
        if (epi.bias) tail.bias = static_cast<const uint16_t*>(epi.bias) + n1;
        tail.out = epi.mode == EPI_F32 ? static_cast<void*>(static_cast<float*>(epi.out) + n1) : static_cast<void*>(static_cast<uint16_t*>(epi.out) + n1);
        return launch_gemm_mfma(A, lda, static_cast<const uint16_t*>(W) + static_cast<int64_t>(n1) * ldw, ldw, M, N - n1, K, tail, st);
      }
    }
  }
  return launch_kind(kind, A, lda, W, ldw, M, N, K, epi, st);
}

}  // namespace speca
