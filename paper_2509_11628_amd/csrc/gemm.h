// Linear layers of the target model:  C[M,N] = A[M,K] * W[N,K]^T (+ bias) with a fused
// epilogue.  A and W are row-major with K contiguous, in the model dtype; accumulation
// is fp32.  Two kernel families implement it: bf16 MFMA with LDS-staged tiles (the dense
// contractions of reference steps) and a plain fp32-FMA tile kernel for fp32 models.
#pragma once

#include "common.h"

namespace speca {

enum EpiMode {
  EPI_STORE = 0,   // out[m][n] = T(acc + bias)
  EPI_GELU = 1,    // out[m][n] = T(gelu_tanh(acc + bias))
  EPI_SILU = 2,    // out[m][n] = T(silu(acc + bias))
  EPI_F32 = 3,     // out[m][n] = float(acc + bias)
  EPI_BRANCH = 4   // F = acc + bias is a cached branch output: optional cache refresh
                   // (D0 <- F, D^o <- (D^{o-1}_new - D^{o-1}_old) * inv_o), then h[m][n] += gate[row][n] * F
};

struct GemmEpi {
  int mode = EPI_STORE;
  const void* bias = nullptr;     // [N] model dtype
  void* out = nullptr;            // STORE/GELU/SILU/F32 destination
  int64_t ldo = 0;
  int shared_chip = 0;            // dispatch hint: this many launches run side by side (row groups of one step on their
                                  // own streams); each is planned for its share of the compute units.  0 or 1: alone
  // EPI_BRANCH
  float* h = nullptr;             // [M][N] fp32 residual stream
  int64_t ldh = 0;
  const float* gate = nullptr;    // gate[(m / tokens) * gate_stride + n]
  int64_t gate_stride = 0;
  int tokens = 1;                 // tokens per row: m = i * tokens + t
  int refresh = 0;                // update cache slot `slot` for rows rt.row[i]
  int slot = 0;
  int64_t cache_elem_offset = 0;  // added to the position inside the cache row (a launch that covers a token sub-range)
  CacheGeom g{};
  RowTable rt{};
};

// M may be ragged; N % 4 == 0 and K % 8 == 0 are required (checked).
Error launch_gemm(int dtype, const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi,
                  hipStream_t st);

// softmax(q k^T / sqrt(hd)) v without mask.  qkv: [rows][T][3][H][hd] (model dtype),
// out: [rows][T][ldo] with the H*hd result in the first columns (ldo >= H*hd, ldo % 4 == 0).
Error launch_attention(int dtype, const void* qkv, void* out, int64_t ldo, int rows, int T, int H, int hd, hipStream_t st);

}  // namespace speca
