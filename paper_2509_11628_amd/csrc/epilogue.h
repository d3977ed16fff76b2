// Device-side epilogues shared by the GEMM kernels.  An epilogue is applied to a quad of
// four consecutive output features (n .. n+3, n % 4 == 0) of one output row m, holding
// fp32 accumulators.
#pragma once

#include "gemm.h"

namespace speca {

// GELU, tanh form, with tanh(u) = 1 - 2 / (1 + exp(2u)) (exact identity; saturates correctly at both ends)
__device__ inline float gelu_tanh_f(float a) {
  const float k = 0.7978845608028654f;   // sqrt(2/pi)
  const float u = k * (a + 0.044715f * a * a * a);
  const float t = 1.0f - __fdividef(2.0f, 1.0f + __expf(2.0f * u));
  return 0.5f * a * (1.0f + t);
}
__device__ inline float silu_f(float a) { return a / (1.0f + __expf(-a)); }

template <typename T> struct Store4;
template <> struct Store4<float> {
  __device__ static void st(float* p, const float* v) { *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]); }
  __device__ static void ld(const float* p, float* v) {
    const float4 r = *reinterpret_cast<const float4*>(p);
    v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
  }
};
template <> struct Store4<bf16_t> {
  __device__ static void st(bf16_t* p, const float* v) {
    uint2 r;
    r.x = static_cast<uint32_t>(f32_to_bf16(v[0])) | (static_cast<uint32_t>(f32_to_bf16(v[1])) << 16);
    r.y = static_cast<uint32_t>(f32_to_bf16(v[2])) | (static_cast<uint32_t>(f32_to_bf16(v[3])) << 16);
    *reinterpret_cast<uint2*>(p) = r;
  }
  __device__ static void ld(const bf16_t* p, float* v) {
    const uint2 r = *reinterpret_cast<const uint2*>(p);
    v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xFFFF0000u);
    v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xFFFF0000u);
  }
};

// T = model / cache storage type.  MODE is a compile-time EpiMode.
template <typename T, int MODE>
__device__ inline void epilogue_quad(const GemmEpi& e, int m, int n, float v[4]) {
  if (e.bias) {
    float b[4];
    Store4<T>::ld(static_cast<const T*>(e.bias) + n, b);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] += b[i];
  }
  if (MODE == EPI_STORE || MODE == EPI_GELU || MODE == EPI_SILU) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (MODE == EPI_GELU) v[i] = gelu_tanh_f(v[i]);
      if (MODE == EPI_SILU) v[i] = silu_f(v[i]);
    }
    Store4<T>::st(static_cast<T*>(e.out) + static_cast<int64_t>(m) * e.ldo + n, v);
  } else if (MODE == EPI_F32) {
    Store4<float>::st(static_cast<float*>(e.out) + static_cast<int64_t>(m) * e.ldo + n, v);
  } else {   // EPI_BRANCH
    const int i = m / e.tokens;
    const int t = m - i * e.tokens;
    if (e.refresh) {
      // Eq. 3 as a recursion on the unrounded new values; each is rounded once when stored
      const int order = e.rt.order[i];
      const int64_t pos = e.cache_elem_offset + static_cast<int64_t>(t) * e.ldh + n;     // ldh == hidden == N for branch outputs
      T* base = static_cast<T*>(e.g.base);
      float cur[4] = {v[0], v[1], v[2], v[3]};
      float old[4];
      if (order >= 1) Store4<T>::ld(base + e.g.offset(e.slot, 0, e.rt.row[i]) + pos, old);
      Store4<T>::st(base + e.g.offset(e.slot, 0, e.rt.row[i]) + pos, cur);
      for (int o = 1; o <= order; ++o) {
        const float inv = e.rt.w[i][o - 1];
        float nxt_old[4];
        T* d = base + e.g.offset(e.slot, o, e.rt.row[i]) + pos;
        if (o < order) Store4<T>::ld(d, nxt_old);
#pragma unroll
        for (int q = 0; q < 4; ++q) cur[q] = (cur[q] - old[q]) * inv;
        Store4<T>::st(d, cur);
#pragma unroll
        for (int q = 0; q < 4; ++q) old[q] = nxt_old[q];
      }
    }
    float g[4], hv[4];
    Store4<float>::ld(e.gate + static_cast<int64_t>(i) * e.gate_stride + n, g);
    float* hp = e.h + static_cast<int64_t>(m) * e.ldh + n;
    Store4<float>::ld(hp, hv);
#pragma unroll
    for (int q = 0; q < 4; ++q) hv[q] = fmaf(g[q], v[q], hv[q]);
    Store4<float>::st(hp, hv);
  }
}

}  // namespace speca
