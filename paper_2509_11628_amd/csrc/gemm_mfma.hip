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
#include "epilogue.h"
#include "gemm.h"

namespace speca {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;
constexpr int LDS_STRIDE = BK + 8;   // elements; 144-byte rows

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // first-class vector: stays in registers

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

  // XCD-aware tile id: blocks b, b+8, b+16, ... run on the same XCD; give them neighbouring tiles
  // (the grid is rounded up to a multiple of 8; surplus blocks leave at once).  Inside an XCD's
  // range tiles are walked in groups of group_m M-panels, N fastest across the group's panels,
  // so that the tiles in flight at one time form a compact rectangle and share operand panels
  // in that XCD's L2.
  const int bid = blockIdx.x;
  const int per_xcd = gridDim.x / 8;
  const int tile = (bid % 8) * per_xcd + bid / 8;
  if (tile >= tiles_m * tiles_n) return;
  int tm, tn;
  {
    const int per_group = group_m * tiles_n;
    const int g = tile / per_group;
    const int first = g * group_m;
    const int h = tiles_m - first < group_m ? tiles_m - first : group_m;
    const int r = tile - g * per_group;
    tm = first + r % h;
    tn = r / h;
  }
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

  // epilogue.  acc[i][j][4*jj + ii] = C[m][n] with m = wm*WM + j*32 + l32, n = wn*WN + i*32 + 8*jj + 4*lhi + ii
  // inside the tile.  The tile goes through LDS once (fp32, rows padded by 16 bytes: conflict-free for
  // the 16-byte writes of 16 consecutive lanes) so that every global access of the epilogue is a
  // contiguous run along n: a half-wave covers one 512-byte (fp32) / 256-byte (bf16) row segment.
  constexpr int CST = BN + 4;                        // floats per staged row
  float* Cs = reinterpret_cast<float*>(smem);        // [BM][CST]; the operand buffers are dead by now
#pragma unroll
  for (int j = 0; j < TM; ++j)
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int r = wm * WM + j * 32 + l32, c = wn * WN + i * 32 + 8 * jj + 4 * lhi;
        *reinterpret_cast<float4*>(Cs + r * CST + c) =
            make_float4(acc[i][j][4 * jj], acc[i][j][4 * jj + 1], acc[i][j][4 * jj + 2], acc[i][j][4 * jj + 3]);
      }
  __syncthreads();
  constexpr int QPR = BN / 4;                        // quads per row
  constexpr int RPP = NT / QPR;                      // rows per pass
  constexpr int PASSES = BM / RPP;
  const int qc = (tid % QPR) * 4, qr = tid / QPR;
  const int n = n0 + qc;
  if (n >= N) return;
  float bias[4] = {0.f, 0.f, 0.f, 0.f};
  if (epi.bias) Store4<bf16_t>::ld(static_cast<const bf16_t*>(epi.bias) + n, bias);
  if (MODE == EPI_BRANCH) {
    // batches of EB rows: all loads of the batch are issued before its first store
    constexpr int EB = PASSES % 4 == 0 ? 4 : (PASSES % 2 == 0 ? 2 : 1);
    const int m_last = (m0 + BM < M ? m0 + BM : M) - 1;
    const int i_first = m0 / epi.tokens;
    if (i_first == m_last / epi.tokens) {
      // the whole tile lies inside one batch row: block-uniform row table, scalar loads
      const BranchRow<bf16_t> br = branch_row<bf16_t>(epi, i_first, m0);
      for (int p0 = 0; p0 < PASSES; p0 += EB) {
        BranchRegs<bf16_t> regs[EB];
#pragma unroll
        for (int u = 0; u < EB; ++u) {
          const int r = qr + (p0 + u) * RPP;
          if (m0 + r < M) branch_load_u<bf16_t>(epi, br, r, m0 + r, n, regs[u]);
        }
#pragma unroll
        for (int u = 0; u < EB; ++u) {
          const int r = qr + (p0 + u) * RPP;
          if (m0 + r < M) {
            const float4 t = *reinterpret_cast<const float4*>(Cs + r * CST + qc);
            const float v[4] = {t.x + bias[0], t.y + bias[1], t.z + bias[2], t.w + bias[3]};
            branch_finish_u<bf16_t>(epi, br, r, m0 + r, n, v, regs[u]);
          }
        }
      }
    } else {
      for (int p0 = 0; p0 < PASSES; p0 += EB) {
        BranchRegs<bf16_t> regs[EB];
#pragma unroll
        for (int u = 0; u < EB; ++u) {
          const int m = m0 + qr + (p0 + u) * RPP;
          if (m < M) branch_load<bf16_t>(epi, m, n, regs[u]);
        }
#pragma unroll
        for (int u = 0; u < EB; ++u) {
          const int r = qr + (p0 + u) * RPP;
          const int m = m0 + r;
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
    for (int r = qr; r < BM; r += RPP) {
      const int m = m0 + r;
      if (m < M) {
        const float4 t = *reinterpret_cast<const float4*>(Cs + r * CST + qc);
        float v[4] = {t.x + bias[0], t.y + bias[1], t.z + bias[2], t.w + bias[3]};
        epilogue_apply<bf16_t, MODE>(epi, m, n, v);
      }
    }
  }
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

Error launch_gemm_mfma(const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi, hipStream_t st) {
  // Tile shapes, from measurements on the reference-step shapes (M = 4096, N 1152..4608):
  //   256x128 with 8 waves (4x2, wave tile 64x64): three quarters of the operand traffic per FLOP of
  //     a 128x128 tile at the same per-wave register cost; best when it still leaves >= 1 tile per
  //     CU-half and, for short K loops, N is not so wide that 128x128 already fills the chip several
  //     times over;
  //   128x128 with 4 waves: the default for everything else that is big enough;
  //   128x64: problems too small to give each CU a tile otherwise.
  const int64_t t128 = static_cast<int64_t>((M + 127) / 128) * ((N + 127) / 128);
  const int64_t t256 = static_cast<int64_t>((M + 255) / 256) * ((N + 127) / 128);
  if (t256 >= 128 && (t128 <= 1024 || (K >= 2048 && t128 >= 2048)) && M >= 256) return launch_tile<256, 128, 4, 2>(A, lda, W, ldw, M, N, K, epi, st);
  if (t128 >= 200) return launch_tile<128, 128, 2, 2>(A, lda, W, ldw, M, N, K, epi, st);
  return launch_tile<128, 64, 2, 2>(A, lda, W, ldw, M, N, K, epi, st);
}

}  // namespace speca
