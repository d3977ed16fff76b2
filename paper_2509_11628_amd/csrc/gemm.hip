// Dispatch of the linear layers and attention to the kernel families (see gemm.h).
#include "gemm.h"

namespace speca {

Error launch_gemm_simple(int dtype, const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi,
                         hipStream_t st);
Error launch_attention_simple(int dtype, const void* qkv, void* out, int64_t ldo, int rows, int T, int H, int hd, hipStream_t st);
bool gemm_mfma_supported(const void* A, int64_t lda, const void* W, int64_t ldw, int N, int K);
Error launch_gemm_mfma(const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi, hipStream_t st);

bool attention_mfma_supported(const void* qkv, const void* out, int64_t ldo, int H, int hd);
Error launch_attention_mfma(const void* qkv, void* out, int64_t ldo, int rows, int T, int H, int hd, hipStream_t st);

Error launch_gemm(int dtype, const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi,
                  hipStream_t st) {
  if (!A || !W) SPECA_FAIL(SPECA_EINVAL, "gemm: NULL operand");
  if (M < 1 || N < 4 || K < 1 || N % 4) SPECA_FAIL(SPECA_EINVAL, "gemm: M=%d N=%d K=%d (N must be a multiple of 4)", M, N, K);
  if (lda < K || ldw < K) SPECA_FAIL(SPECA_EINVAL, "gemm: leading dimensions smaller than K");
  if (epi.mode == EPI_BRANCH) {
    if (!epi.h || !epi.gate || epi.tokens < 1 || epi.ldh != N) SPECA_FAIL(SPECA_EINVAL, "gemm: branch epilogue arguments");
    if (M % epi.tokens) SPECA_FAIL(SPECA_EINVAL, "gemm: M=%d is not a multiple of tokens=%d", M, epi.tokens);
    if (epi.refresh) {
      if (M / epi.tokens != epi.rt.n || epi.cache_elem_offset < 0 || epi.cache_elem_offset % 4 ||
          epi.g.E < epi.cache_elem_offset + static_cast<int64_t>(epi.tokens) * N || epi.slot < 0 || epi.slot >= epi.g.n_slots)
        SPECA_FAIL(SPECA_EINVAL, "gemm: cache refresh geometry does not match the launch");
      for (int i = 0; i < epi.rt.n; ++i)
        if (epi.rt.row[i] < 0 || epi.rt.order[i] < 0 || epi.rt.row[i] / epi.g.batch_rows + epi.rt.order[i] > epi.g.m)   // plane + order
          SPECA_FAIL(SPECA_EINVAL, "gemm: cache row table out of range");
    }
  } else if (!epi.out || epi.ldo < N) {
    SPECA_FAIL(SPECA_EINVAL, "gemm: output missing");
  }
  if (dtype == SPECA_BF16 && gemm_mfma_supported(A, lda, W, ldw, N, K))
    return launch_gemm_mfma(A, lda, W, ldw, M, N, K, epi, st);
  return launch_gemm_simple(dtype, A, lda, W, ldw, M, N, K, epi, st);
}

Error launch_attention(int dtype, const void* qkv, void* out, int64_t ldo, int rows, int T, int H, int hd, hipStream_t st) {
  if (!qkv || !out || rows < 1 || T < 1 || H < 1 || ldo < static_cast<int64_t>(H) * hd || ldo % 4) SPECA_FAIL(SPECA_EINVAL, "attention: bad arguments");
  if (dtype == SPECA_BF16 && attention_mfma_supported(qkv, out, ldo, H, hd))
    return launch_attention_mfma(qkv, out, ldo, rows, T, H, hd, st);
  return launch_attention_simple(dtype, qkv, out, ldo, rows, T, H, hd, st);
}

}  // namespace speca
