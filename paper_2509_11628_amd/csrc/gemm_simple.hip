// Plain fp32-FMA tile kernels: the linear layers and attention of fp32 models (there is
// no fp32 path through the bf16 matrix cores), and of shapes the MFMA kernels do not take.
// 64x64 output tile per 256-thread block, K staged through LDS in steps of 16, each
// thread owns a 4x4 micro-tile.  K is walked in order, so a row's result does not depend
// on M or on which other rows share the launch.
#include "epilogue.h"
#include "gemm.h"

namespace speca {

namespace {

template <typename T> __device__ inline float ld_as_f32(const T* p);
template <> __device__ inline float ld_as_f32<float>(const float* p) { return *p; }
template <> __device__ inline float ld_as_f32<bf16_t>(const bf16_t* p) { return bf16_to_f32(p->bits); }

constexpr int TM = 64, TN = 64, TK = 16;

template <typename T, int MODE>
__global__ __launch_bounds__(256) void gemm_simple_kernel(const T* __restrict__ A, int64_t lda, const T* __restrict__ W, int64_t ldw,
                                                          int M, int N, int K, GemmEpi epi) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Ws[TK][TN + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  const int tx = tid & 15, ty = tid >> 4;           // tx -> n quad, ty -> m quad
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;
  for (int k0 = 0; k0 < K; k0 += TK) {
    // 64 rows x 16 k = 1024 elements per operand, 4 per thread
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int idx = tid + r * 256;
      const int row = idx >> 4, kk = idx & 15;
      const int k = k0 + kk;
      float a = 0.0f, w = 0.0f;
      if (k < K) {
        if (m0 + row < M) a = ld_as_f32(A + static_cast<int64_t>(m0 + row) * lda + k);
        if (n0 + row < N) w = ld_as_f32(W + static_cast<int64_t>(n0 + row) * ldw + k);
      }
      As[kk][row] = a;
      Ws[kk][row] = w;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = Ws[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
  const int n = n0 + tx * 4;
  if (n < N) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + ty * 4 + i;
      if (m < M) epilogue_quad<T, MODE>(epi, m, n, acc[i]);
    }
  }
}

template <typename T>
Error launch_simple_t(const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi, hipStream_t st) {
  dim3 grid((N + TN - 1) / TN, (M + TM - 1) / TM);
  const T* a = static_cast<const T*>(A);
  const T* w = static_cast<const T*>(W);
  switch (epi.mode) {
    case EPI_STORE: gemm_simple_kernel<T, EPI_STORE><<<grid, 256, 0, st>>>(a, lda, w, ldw, M, N, K, epi); break;
    case EPI_GELU: gemm_simple_kernel<T, EPI_GELU><<<grid, 256, 0, st>>>(a, lda, w, ldw, M, N, K, epi); break;
    case EPI_SILU: gemm_simple_kernel<T, EPI_SILU><<<grid, 256, 0, st>>>(a, lda, w, ldw, M, N, K, epi); break;
    case EPI_F32: gemm_simple_kernel<T, EPI_F32><<<grid, 256, 0, st>>>(a, lda, w, ldw, M, N, K, epi); break;
    case EPI_BRANCH: gemm_simple_kernel<T, EPI_BRANCH><<<grid, 256, 0, st>>>(a, lda, w, ldw, M, N, K, epi); break;
    default: SPECA_FAIL(SPECA_EINVAL, "gemm: epilogue mode %d", epi.mode);
  }
  SPECA_HIP(hipGetLastError());
  return ok();
}

// ---------------------------------------------------------------------------------------
// Attention, one thread per query, keys/values staged through LDS in tiles of 64, online
// softmax in fp32.  hd <= 128.
constexpr int AT_Q = 64;      // queries per block
constexpr int AT_K = 32;      // keys per LDS tile
constexpr int HD_MAX = 128;

template <typename T, int HD>
__global__ __launch_bounds__(AT_Q) void attention_simple_kernel(const T* __restrict__ qkv, T* __restrict__ out, int64_t ldo, int Tn,
                                                                int H, float scale) {
  __shared__ float Ks[AT_K][HD];
  __shared__ float Vs[AT_K][HD];
  const int row = blockIdx.z, head = blockIdx.y;
  const int qi = blockIdx.x * AT_Q + threadIdx.x;
  const int64_t D = static_cast<int64_t>(H) * HD;
  const T* base = qkv + static_cast<int64_t>(row) * Tn * 3 * D;
  float q[HD], o[HD];
  const bool live = qi < Tn;
#pragma unroll
  for (int d = 0; d < HD; ++d) {
    q[d] = live ? ld_as_f32(base + static_cast<int64_t>(qi) * 3 * D + head * HD + d) * scale : 0.0f;
    o[d] = 0.0f;
  }
  float mx = -INFINITY, sum = 0.0f;
  for (int k0 = 0; k0 < Tn; k0 += AT_K) {
    const int nk = Tn - k0 < AT_K ? Tn - k0 : AT_K;
    for (int idx = threadIdx.x; idx < AT_K * HD; idx += AT_Q) {
      const int kk = idx / HD, d = idx - kk * HD;
      float kv = 0.0f, vv = 0.0f;
      if (kk < nk) {
        const T* p = base + static_cast<int64_t>(k0 + kk) * 3 * D + head * HD + d;
        kv = ld_as_f32(p + D);
        vv = ld_as_f32(p + 2 * D);
      }
      Ks[kk][d] = kv;
      Vs[kk][d] = vv;
    }
    __syncthreads();
    for (int kk = 0; kk < nk; ++kk) {
      float s = 0.0f;
#pragma unroll
      for (int d = 0; d < HD; ++d) s = fmaf(q[d], Ks[kk][d], s);
      const float nm = fmaxf(mx, s);
      const float corr = __expf(mx - nm);
      const float p = __expf(s - nm);
      sum = sum * corr + p;
#pragma unroll
      for (int d = 0; d < HD; ++d) o[d] = fmaf(p, Vs[kk][d], o[d] * corr);
      mx = nm;
    }
    __syncthreads();
  }
  if (live) {
    const float inv = 1.0f / sum;
    T* op = out + (static_cast<int64_t>(row) * Tn + qi) * ldo + head * HD;
#pragma unroll
    for (int d = 0; d < HD; ++d) {
      if (sizeof(T) == 2) reinterpret_cast<uint16_t*>(op)[d] = f32_to_bf16(o[d] * inv);
      else reinterpret_cast<float*>(op)[d] = o[d] * inv;
    }
  }
}

template <typename T, int HD>
Error launch_attn_t(const void* qkv, void* out, int64_t ldo, int rows, int Tn, int H, hipStream_t st) {
  dim3 grid((Tn + AT_Q - 1) / AT_Q, H, rows);
  attention_simple_kernel<T, HD><<<grid, AT_Q, 0, st>>>(static_cast<const T*>(qkv), static_cast<T*>(out), ldo, Tn, H,
                                                        1.0f / sqrtf(static_cast<float>(HD)));
  SPECA_HIP(hipGetLastError());
  return ok();
}

template <typename T>
Error launch_attn_hd(const void* qkv, void* out, int64_t ldo, int rows, int Tn, int H, int hd, hipStream_t st) {
  switch (hd) {
    case 16: return launch_attn_t<T, 16>(qkv, out, ldo, rows, Tn, H, st);
    case 32: return launch_attn_t<T, 32>(qkv, out, ldo, rows, Tn, H, st);
    case 64: return launch_attn_t<T, 64>(qkv, out, ldo, rows, Tn, H, st);
    case 72: return launch_attn_t<T, 72>(qkv, out, ldo, rows, Tn, H, st);
    case 128: return launch_attn_t<T, 128>(qkv, out, ldo, rows, Tn, H, st);
  }
  SPECA_FAIL(SPECA_EUNSUPPORTED, "attention: head_dim %d (supported: 16, 32, 64, 72, 128)", hd);
}

}  // namespace

Error launch_gemm_simple(int dtype, const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, const GemmEpi& epi,
                         hipStream_t st) {
  return dtype == SPECA_BF16 ? launch_simple_t<bf16_t>(A, lda, W, ldw, M, N, K, epi, st)
                             : launch_simple_t<float>(A, lda, W, ldw, M, N, K, epi, st);
}

Error launch_attention_simple(int dtype, const void* qkv, void* out, int64_t ldo, int rows, int T, int H, int hd, hipStream_t st) {
  return dtype == SPECA_BF16 ? launch_attn_hd<bf16_t>(qkv, out, ldo, rows, T, H, hd, st) : launch_attn_hd<float>(qkv, out, ldo, rows, T, H, hd, st);
}

}  // namespace speca
