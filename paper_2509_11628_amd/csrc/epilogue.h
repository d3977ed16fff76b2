// Device-side epilogues shared by the GEMM kernels.  An epilogue is applied to a quad of
// four consecutive output features (n .. n+3, n % 4 == 0) of one output row m, holding
// fp32 accumulators.
#pragma once

#include "gemm.h"

namespace speca {

// GELU, tanh form.  0.5 a (1 + tanh u) = a / (1 + exp(-2u)) with u = sqrt(2/pi) (a + 0.044715 a^3) (exact
// identity; saturates correctly at both ends: exp2 -> 0 gives a, exp2 -> inf gives a * 0).  The constants
// fold -2 sqrt(2/pi) log2(e) into the cubic so the body is 5 full-rate operations around one hardware
// exp2 and one hardware reciprocal (each about 1 ulp): the epilogue of the wide MLP GEMM is ALU time
// that nothing overlaps, and the libm-style exp / divide took twice as long there.
__device__ inline float gelu_tanh_f(float a) {
  const float c1 = -2.3022082f;            // -2 sqrt(2/pi) log2(e)
  const float c2 = -0.10294324f;           // c1 * 0.044715
  const float a2 = a * a;
  const float w = a * fmaf(c2, a2, c1);
  return a * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(w));
}
__device__ inline float silu_f(float a) { return a * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950409f * a)); }

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

// Streaming forms for data that is written once and read a whole step later (the cache): no reuse to
// keep in L2.
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ inline void st4_stream(bf16_t* p, const float* v) {
  u32x2_t r;
  r.x = static_cast<uint32_t>(f32_to_bf16(v[0])) | (static_cast<uint32_t>(f32_to_bf16(v[1])) << 16);
  r.y = static_cast<uint32_t>(f32_to_bf16(v[2])) | (static_cast<uint32_t>(f32_to_bf16(v[3])) << 16);
  __builtin_nontemporal_store(r, reinterpret_cast<u32x2_t*>(p));
}
__device__ inline void st4_stream(float* p, const float* v) {
  f32x4_t r = {v[0], v[1], v[2], v[3]};
  __builtin_nontemporal_store(r, reinterpret_cast<f32x4_t*>(p));
}
__device__ inline void ld4_stream(const bf16_t* p, float* v) {
  const u32x2_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
  v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xFFFF0000u);
  v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xFFFF0000u);
}
__device__ inline void ld4_stream(const float* p, float* v) {
  const f32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
  v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
}

template <typename T, int MODE>
__device__ inline void epilogue_apply(const GemmEpi& e, int m, int n, float v[4]);

// T = model / cache storage type.  MODE is a compile-time EpiMode.
template <typename T, int MODE>
__device__ inline void epilogue_quad(const GemmEpi& e, int m, int n, float v[4]) {
  if (e.bias) {
    float b[4];
    Store4<T>::ld(static_cast<const T*>(e.bias) + n, b);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] += b[i];
  }
  epilogue_apply<T, MODE>(e, m, n, v);
}

// The epilogue after the bias has been added.
template <typename T, int MODE>
__device__ inline void epilogue_apply(const GemmEpi& e, int m, int n, float v[4]) {
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


// ---- two-phase form of the branch epilogue --------------------------------------------------
// The GEMM kernels apply the branch epilogue to several rows per thread.  Done row by row,
// every row costs a full memory latency (load old differences / residual -> compute -> store).
// Splitting it into a load phase and a finish phase lets a thread put the loads of a whole
// batch of rows in flight before the first store.
template <typename T>
struct BranchRegs {
  float old[SPECA_MAX_ORDER][4];   // D^0 .. D^{order-1} before the refresh
  float g[4], hv[4];
};

template <typename T>
__device__ inline void branch_load(const GemmEpi& e, int m, int n, BranchRegs<T>& r) {
  const int i = m / e.tokens;
  const int t = m - i * e.tokens;
  if (e.refresh) {
    const int order = e.rt.order[i];
    const int64_t pos = e.cache_elem_offset + static_cast<int64_t>(t) * e.ldh + n;
    const T* base = static_cast<const T*>(e.g.base);
#pragma unroll
    for (int o = 0; o < SPECA_MAX_ORDER; ++o)
      if (o < order) Store4<T>::ld(base + e.g.offset(e.slot, o, e.rt.row[i]) + pos, r.old[o]);
  }
  Store4<float>::ld(e.gate + static_cast<int64_t>(i) * e.gate_stride + n, r.g);
  Store4<float>::ld(e.h + static_cast<int64_t>(m) * e.ldh + n, r.hv);
}

// v = accumulators + bias (already added by the caller)
template <typename T>
__device__ inline void branch_finish(const GemmEpi& e, int m, int n, const float v[4], BranchRegs<T>& r) {
  const int i = m / e.tokens;
  const int t = m - i * e.tokens;
  if (e.refresh) {
    const int order = e.rt.order[i];
    const int64_t pos = e.cache_elem_offset + static_cast<int64_t>(t) * e.ldh + n;
    T* base = static_cast<T*>(e.g.base);
    float cur[4] = {v[0], v[1], v[2], v[3]};
    Store4<T>::st(base + e.g.offset(e.slot, 0, e.rt.row[i]) + pos, cur);
#pragma unroll
    for (int o = 1; o <= SPECA_MAX_ORDER; ++o)
      if (o <= order) {
        const float inv = e.rt.w[i][o - 1];
#pragma unroll
        for (int q = 0; q < 4; ++q) cur[q] = (cur[q] - r.old[o - 1][q]) * inv;
        Store4<T>::st(base + e.g.offset(e.slot, o, e.rt.row[i]) + pos, cur);
      }
  }
  float hv[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) hv[q] = fmaf(r.g[q], v[q], r.hv[q]);
  Store4<float>::st(e.h + static_cast<int64_t>(m) * e.ldh + n, hv);
}


// ---- block-uniform form ------------------------------------------------------------------------
// When all rows of a tile belong to one batch row, the row table lookup (cache row, order,
// reciprocal divisors) is the same for the whole block: it is read once through scalar loads and
// the per-quad work needs no table access in front of its cache loads.
template <typename T>
struct BranchRow {
  int order;                         // differences to refresh (0 when refresh is off)
  bool refresh;
  float inv[SPECA_MAX_ORDER];
  T* d[SPECA_MAX_ORDER + 1];         // D^o of (slot, cache row), already offset by cache_elem_offset
  const float* gate;
  int t0;                            // token index of tile row 0 inside the batch row
};

template <typename T>
__device__ inline BranchRow<T> branch_row(const GemmEpi& e, int i, int m0) {
  BranchRow<T> b;
  b.refresh = e.refresh != 0;
  b.order = b.refresh ? e.rt.order[i] : 0;
  T* base = static_cast<T*>(e.g.base);
#pragma unroll
  for (int o = 0; o <= SPECA_MAX_ORDER; ++o)
    b.d[o] = (b.refresh && o <= b.order) ? base + e.g.offset(e.slot, o, e.rt.row[i]) + e.cache_elem_offset : base;
#pragma unroll
  for (int o = 0; o < SPECA_MAX_ORDER; ++o) b.inv[o] = (b.refresh && o < b.order) ? e.rt.w[i][o] : 0.0f;
  b.gate = e.gate + static_cast<int64_t>(i) * e.gate_stride;
  b.t0 = m0 - i * e.tokens;
  return b;
}

template <typename T>
__device__ inline void branch_load_u(const GemmEpi& e, const BranchRow<T>& b, int r, int m, int n, BranchRegs<T>& regs) {
  const int64_t pos = static_cast<int64_t>(b.t0 + r) * e.ldh + n;
#pragma unroll
  for (int o = 0; o < SPECA_MAX_ORDER; ++o)
    if (o < b.order) ld4_stream(b.d[o] + pos, regs.old[o]);
  Store4<float>::ld(e.h + static_cast<int64_t>(m) * e.ldh + n, regs.hv);    // the gate is per (batch row, n): the caller holds it
}

template <typename T>
__device__ inline void branch_finish_u(const GemmEpi& e, const BranchRow<T>& b, int r, int m, int n, const float v[4], const float g[4],
                                       BranchRegs<T>& regs) {
  if (b.refresh) {
    const int64_t pos = static_cast<int64_t>(b.t0 + r) * e.ldh + n;
    float cur[4] = {v[0], v[1], v[2], v[3]};
    st4_stream(b.d[0] + pos, cur);
#pragma unroll
    for (int o = 1; o <= SPECA_MAX_ORDER; ++o)
      if (o <= b.order) {
        const float inv = b.inv[o - 1];
#pragma unroll
        for (int q = 0; q < 4; ++q) cur[q] = (cur[q] - regs.old[o - 1][q]) * inv;
        st4_stream(b.d[o] + pos, cur);
      }
  }
  float hv[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) hv[q] = fmaf(g[q], v[q], regs.hv[q]);
  Store4<float>::st(e.h + static_cast<int64_t>(m) * e.ldh + n, hv);
}

}  // namespace speca
