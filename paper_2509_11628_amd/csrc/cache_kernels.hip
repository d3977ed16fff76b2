// HBM-bound kernels of the SpeCa cache for gfx950: difference refresh (Eq. 3 as a
// recursion), Taylor forecast (Eq. 2), fused forecast-and-fold into the hidden state,
// and the relative-error reductions of the verifier (Eq. 4).
//
// All of them stream the cache once with 128-bit accesses and do their arithmetic in
// fp32 on the vector ALUs; there is no contraction here, so no MFMA.  A thread owns
// 16 bytes of every tensor it touches (8 bf16 or 4 fp32 values); a block of 256 threads
// covers kUnroll such vectors per thread.  Reductions use a fixed order (per-thread
// sequence, wave shuffle tree, per-block LDS order, second pass over fixed-size chunk
// partials), so results are bit-reproducible and do not depend on which other rows share
// the launch.

#include "kernels.h"

namespace speca {

namespace {

constexpr int kThreads = 256;

template <typename T> struct Vec;
template <> struct Vec<float> {
  static constexpr int N = 4;
  using raw = float4;
  __device__ static void unpack(const raw& r, float* f) { f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w; }
  __device__ static raw pack(const float* f) { return make_float4(f[0], f[1], f[2], f[3]); }
  __device__ static float load1(const float* p) { return *p; }
  __device__ static void store1(float* p, float v) { *p = v; }
};
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  using raw = uint4;
  __device__ static void unpack(const raw& r, float* f) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  __device__ static raw pack(const float* f) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = static_cast<uint32_t>(f32_to_bf16(f[2 * i])) | (static_cast<uint32_t>(f32_to_bf16(f[2 * i + 1])) << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
  }
  __device__ static float load1(const bf16_t* p) { return bf16_to_f32(p->bits); }
  __device__ static void store1(bf16_t* p, float v) { p->bits = f32_to_bf16(v); }
};

template <typename T>
__device__ inline typename Vec<T>::raw ldg(const T* p) {
  return *reinterpret_cast<const typename Vec<T>::raw*>(p);
}
// 16-byte streaming forms: the cache planes and the materialised forecast are touched once per step and are far
// larger than any cache level, so they are marked non-temporal (measured +2..3 % on the forecast kernels).
typedef unsigned int stream_u32x4 __attribute__((ext_vector_type(4)));
template <typename T>
__device__ inline typename Vec<T>::raw ldg_stream(const T* p) {
  const stream_u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const stream_u32x4*>(p));
  typename Vec<T>::raw o;
  __builtin_memcpy(&o, &r, 16);
  return o;
}
template <typename T>
__device__ inline void stg_stream(T* p, const typename Vec<T>::raw& v) {
  stream_u32x4 r;
  __builtin_memcpy(&r, &v, 16);
  __builtin_nontemporal_store(r, reinterpret_cast<stream_u32x4*>(p));
}
template <typename T>
__device__ inline void stg(T* p, const typename Vec<T>::raw& v) {
  *reinterpret_cast<typename Vec<T>::raw*>(p) = v;
}

// ---------------------------------------------------------------------------------------
// Forecast, materialised:  out[slot][i][e] = sum_{o<=order_i} c[i][o] * D^o[slot][row_i][e]
// grid = (chunks of E, n_rows, n_slots)
template <typename T, int NT, bool VEC>
__global__ __launch_bounds__(kThreads) void forecast_kernel(CacheGeom g, RowTable rt, T* __restrict__ out) {
  const int i = blockIdx.y, slot = blockIdx.z;
  const int row = rt.row[i];
  const int order = rt.order[i];
  float c[NT];
#pragma unroll
  for (int o = 0; o < NT; ++o) c[o] = (o <= order) ? rt.w[i][o] : 0.0f;
  const T* base = static_cast<const T*>(g.base);
  const T* src[NT];
#pragma unroll
  for (int o = 0; o < NT; ++o) src[o] = base + g.offset(slot, o <= order ? o : 0, row);
  T* dst = out + (static_cast<int64_t>(slot) * rt.n + i) * g.E;
  constexpr int V = Vec<T>::N;
  if (VEC) {
    const int64_t nvec = g.E / V;
    for (int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; v < nvec;
         v += static_cast<int64_t>(gridDim.x) * kThreads) {
      typename Vec<T>::raw r[NT];
#pragma unroll
      for (int o = 0; o < NT; ++o)
        if (o <= order) r[o] = ldg_stream(src[o] + v * V);
      float acc[V];
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] = 0.0f;
#pragma unroll
      for (int o = 0; o < NT; ++o)
        if (o <= order) {
          float f[V];
          Vec<T>::unpack(r[o], f);
#pragma unroll
          for (int e = 0; e < V; ++e) acc[e] = fmaf(c[o], f[e], acc[e]);
        }
      stg_stream(dst + v * V, Vec<T>::pack(acc));
    }
  } else {
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; e < g.E;
         e += static_cast<int64_t>(gridDim.x) * kThreads) {
      float acc = 0.0f;
#pragma unroll
      for (int o = 0; o < NT; ++o)
        if (o <= order) acc = fmaf(c[o], Vec<T>::load1(src[o] + e), acc);
      Vec<T>::store1(dst + e, acc);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Refresh from materialised features:  D0 <- F;  D^o <- (D^{o-1}_new - D^{o-1}_old) * inv_o.
// The recursion runs on the unrounded new values; each is rounded once when stored.
// rt.order[i] = order after the refresh (min(m, #references before)); rt.w[i][o-1] = 1/d_o.
template <typename T, int NT, bool VEC>
__global__ __launch_bounds__(kThreads) void refresh_kernel(CacheGeom g, RowTable rt, const T* __restrict__ feat) {
  const int i = blockIdx.y, slot = blockIdx.z;
  const int row = rt.row[i];
  const int order = rt.order[i];
  T* base = static_cast<T*>(g.base);
  T* d[NT];
#pragma unroll
  for (int o = 0; o < NT; ++o) d[o] = base + g.offset(slot, o <= order ? o : 0, row);
  const T* f = feat + (static_cast<int64_t>(slot) * rt.n + i) * g.E;
  constexpr int V = Vec<T>::N;
  if (VEC) {
    const int64_t nvec = g.E / V;
    for (int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; v < nvec;
         v += static_cast<int64_t>(gridDim.x) * kThreads) {
      typename Vec<T>::raw rf = ldg_stream(f + v * V);
      typename Vec<T>::raw ro[NT];
#pragma unroll
      for (int o = 0; o + 1 < NT; ++o)
        if (o < order) ro[o] = ldg_stream(d[o] + v * V);
      float cur[V];
      Vec<T>::unpack(rf, cur);
      stg_stream(d[0] + v * V, rf);
#pragma unroll
      for (int o = 1; o < NT; ++o)
        if (o <= order) {
          float old[V];
          Vec<T>::unpack(ro[o - 1], old);
          const float inv = rt.w[i][o - 1];
#pragma unroll
          for (int e = 0; e < V; ++e) cur[e] = (cur[e] - old[e]) * inv;
          stg_stream(d[o] + v * V, Vec<T>::pack(cur));
        }
    }
  } else {
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; e < g.E;
         e += static_cast<int64_t>(gridDim.x) * kThreads) {
      float cur = Vec<T>::load1(f + e);
      float old[NT];
#pragma unroll
      for (int o = 0; o + 1 < NT; ++o)
        if (o < order) old[o] = Vec<T>::load1(d[o] + e);
      Vec<T>::store1(d[0] + e, cur);
#pragma unroll
      for (int o = 1; o < NT; ++o)
        if (o <= order) {
          cur = (cur - old[o - 1]) * rt.w[i][o - 1];
          Vec<T>::store1(d[o] + e, cur);
        }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Verification reductions.  Stage 1: one block per (chunk of kChunk elements, row) writes
// three partial accumulators; stage 2: one wave per row folds the partials and applies the
// metric.  PRED_CACHE: the prediction is not read from memory but formed on the fly from the
// cached differences of one slot (Eq. 2 fused into Eq. 4).
constexpr int kChunk = kThreads * 32;   // elements per stage-1 block, independent of the launch

template <int METRIC>
__device__ inline void acc_update(float p, float t, float& a0, float& a1, float& a2) {
  const float d = p - t;
  if (METRIC == SPECA_METRIC_L2) { a0 = fmaf(d, d, a0); a1 = fmaf(t, t, a1); }
  else if (METRIC == SPECA_METRIC_L1) { a0 += fabsf(d); a1 += fabsf(t); }
  else if (METRIC == SPECA_METRIC_LINF) { a0 = fmaxf(a0, fabsf(d)); a1 = fmaxf(a1, fabsf(t)); }
  else { a0 = fmaf(p, t, a0); a1 = fmaf(t, t, a1); a2 = fmaf(p, p, a2); }
}
template <int METRIC>
__device__ inline float acc_merge(float a, float b) { return METRIC == SPECA_METRIC_LINF ? fmaxf(a, b) : a + b; }

template <int METRIC>
__device__ inline void block_reduce3(float& a0, float& a1, float& a2) {
  // wave64 butterfly, then waves in index order
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    a0 = acc_merge<METRIC>(a0, __shfl_xor(a0, off, 64));
    a1 = acc_merge<METRIC>(a1, __shfl_xor(a1, off, 64));
    a2 = acc_merge<METRIC>(a2, __shfl_xor(a2, off, 64));
  }
  __shared__ float s[3][kThreads / 64];
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { s[0][wave] = a0; s[1][wave] = a1; s[2][wave] = a2; }
  __syncthreads();
  if (threadIdx.x == 0) {
    a0 = s[0][0]; a1 = s[1][0]; a2 = s[2][0];
    for (int w = 1; w < kThreads / 64; ++w) {
      a0 = acc_merge<METRIC>(a0, s[0][w]);
      a1 = acc_merge<METRIC>(a1, s[1][w]);
      a2 = acc_merge<METRIC>(a2, s[2][w]);
    }
  }
}

template <typename T, typename TT, int METRIC, bool PRED_CACHE, int NT, bool VEC>
__global__ __launch_bounds__(kThreads) void verify_partial_kernel(const T* __restrict__ pred, const TT* __restrict__ truth,
                                                                   int64_t E, CacheGeom g, RowTable rt, int slot,
                                                                   float* __restrict__ partial, int n_chunks) {
  const int i = blockIdx.y;
  const int64_t begin = static_cast<int64_t>(blockIdx.x) * kChunk;
  const int64_t end = begin + kChunk < E ? begin + kChunk : E;
  float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f;
  const TT* t = truth + static_cast<int64_t>(i) * E;
  const T* p[NT];
  float c[NT];
  int order = 0;
  if (PRED_CACHE) {
    order = rt.order[i];
    const T* base = static_cast<const T*>(g.base);
#pragma unroll
    for (int o = 0; o < NT; ++o) {
      p[o] = base + g.offset(slot, o <= order ? o : 0, rt.row[i]);
      c[o] = o <= order ? rt.w[i][o] : 0.0f;
    }
  } else {
    p[0] = pred + static_cast<int64_t>(i) * E;
    c[0] = 1.0f;
  }
  if (VEC) {
    // T and TT may differ in width: walk in units of 8 elements
    constexpr int V = 8;
    auto one = [&](int64_t e) {
      float tv[V], pv[V];
      if (sizeof(TT) == 2) {
        Vec<bf16_t>::unpack(*reinterpret_cast<const uint4*>(t + e), tv);
      } else {
        Vec<float>::unpack(*reinterpret_cast<const float4*>(t + e), tv);
        Vec<float>::unpack(*reinterpret_cast<const float4*>(t + e + 4), tv + 4);
      }
#pragma unroll
      for (int q = 0; q < V; ++q) pv[q] = 0.0f;
#pragma unroll
      for (int o = 0; o < NT; ++o)
        if (o <= order) {
          float f[V];
          if (sizeof(T) == 2) {
            Vec<bf16_t>::unpack(*reinterpret_cast<const uint4*>(p[o] + e), f);
          } else {
            Vec<float>::unpack(*reinterpret_cast<const float4*>(p[o] + e), f);
            Vec<float>::unpack(*reinterpret_cast<const float4*>(p[o] + e + 4), f + 4);
          }
#pragma unroll
          for (int q = 0; q < V; ++q) pv[q] = PRED_CACHE ? fmaf(c[o], f[q], pv[q]) : f[q];
        }
#pragma unroll
      for (int q = 0; q < V; ++q) acc_update<METRIC>(pv[q], tv[q], a0, a1, a2);
    };
    if (end - begin == kChunk) {
      // a whole chunk: fixed trip count, so the loads of all trips are in flight before the first sum (same order of sums)
#pragma unroll
      for (int it = 0; it < kChunk / (kThreads * V); ++it) one(begin + (static_cast<int64_t>(it) * kThreads + threadIdx.x) * V);
    } else {
      for (int64_t e = begin + static_cast<int64_t>(threadIdx.x) * V; e < end; e += kThreads * V) one(e);
    }
  } else {
    for (int64_t e = begin + threadIdx.x; e < end; e += kThreads) {
      float pv = 0.0f;
#pragma unroll
      for (int o = 0; o < NT; ++o)
        if (o <= order) {
          const float f = sizeof(T) == 2 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(p[o])[e])
                                         : reinterpret_cast<const float*>(p[o])[e];
          pv = PRED_CACHE ? fmaf(c[o], f, pv) : f;
        }
      const float tv = sizeof(TT) == 2 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(t)[e])
                                       : reinterpret_cast<const float*>(t)[e];
      acc_update<METRIC>(pv, tv, a0, a1, a2);
    }
  }
  block_reduce3<METRIC>(a0, a1, a2);
  if (threadIdx.x == 0) {
    float* o = partial + (static_cast<int64_t>(i) * n_chunks + blockIdx.x) * 3;
    o[0] = a0; o[1] = a1; o[2] = a2;
  }
}

// Stage 2: one wave per row; lane l sums partials l, l+64, ... in order, then butterfly.
template <int METRIC>
__global__ __launch_bounds__(64) void verify_final_kernel(const float* __restrict__ partial, int n_chunks, float eps,
                                                          const float* __restrict__ tau, float* __restrict__ err,
                                                          uint8_t* __restrict__ accept) {
  const int i = blockIdx.x;
  float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f;
  for (int c = threadIdx.x; c < n_chunks; c += 64) {
    const float* p = partial + (static_cast<int64_t>(i) * n_chunks + c) * 3;
    a0 = acc_merge<METRIC>(a0, p[0]);
    a1 = acc_merge<METRIC>(a1, p[1]);
    a2 = acc_merge<METRIC>(a2, p[2]);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    a0 = acc_merge<METRIC>(a0, __shfl_xor(a0, off, 64));
    a1 = acc_merge<METRIC>(a1, __shfl_xor(a1, off, 64));
    a2 = acc_merge<METRIC>(a2, __shfl_xor(a2, off, 64));
  }
  if (threadIdx.x == 0) {
    float e;
    if (METRIC == SPECA_METRIC_L2) e = sqrtf(a0) / (sqrtf(a1) + eps);
    else if (METRIC == SPECA_METRIC_COSINE) e = 1.0f - a0 / (sqrtf(a2) * sqrtf(a1) + eps);
    else e = a0 / (a1 + eps);
    err[i] = e;
    if (tau) accept[i] = e <= tau[i] ? 1 : 0;
  }
}

inline int grid_x_for(int64_t E, int per_thread) {
  int64_t per_block = static_cast<int64_t>(kThreads) * per_thread;
  int64_t gx = (E + per_block - 1) / per_block;
  if (gx < 1) gx = 1;
  if (gx > 65535) gx = 65535;
  return static_cast<int>(gx);
}

template <typename T>
bool aligned_for_vec(const void* p, int64_t E) {
  return (reinterpret_cast<uintptr_t>(p) % 16 == 0) && (E % 8 == 0);
}

}  // namespace

// ---------------------------------------------------------------------------------------
// host launchers

template <typename T, int NT>
static Error launch_forecast_t(const CacheGeom& g, const RowTable& rt, void* out, hipStream_t st) {
  const bool vec = aligned_for_vec<T>(g.base, g.E) && aligned_for_vec<T>(out, g.E);
  // 2 vectors per thread per tensor keeps >= 2 x 16 B loads in flight per tensor
  dim3 grid(grid_x_for(g.E, Vec<T>::N * 2), rt.n, g.n_slots);
  if (vec) forecast_kernel<T, NT, true><<<grid, kThreads, 0, st>>>(g, rt, static_cast<T*>(out));
  else forecast_kernel<T, NT, false><<<grid, kThreads, 0, st>>>(g, rt, static_cast<T*>(out));
  SPECA_HIP(hipGetLastError());
  return ok();
}

template <typename T>
static Error launch_forecast_nt(const CacheGeom& g, const RowTable& rt, void* out, hipStream_t st) {
  int mo = 0;
  for (int i = 0; i < rt.n; ++i) mo = rt.order[i] > mo ? rt.order[i] : mo;
  switch (mo) {
    case 0: return launch_forecast_t<T, 1>(g, rt, out, st);
    case 1: return launch_forecast_t<T, 2>(g, rt, out, st);
    case 2: return launch_forecast_t<T, 3>(g, rt, out, st);
    case 3: return launch_forecast_t<T, 4>(g, rt, out, st);
    default: return launch_forecast_t<T, 5>(g, rt, out, st);
  }
}

Error launch_forecast(const CacheGeom& g, const RowTable& rt, void* out, hipStream_t st) {
  if (rt.n <= 0 || rt.n > kMaxRows) SPECA_FAIL(SPECA_EINVAL, "forecast: %d rows in one launch", rt.n);
  return g.dtype == SPECA_BF16 ? launch_forecast_nt<bf16_t>(g, rt, out, st) : launch_forecast_nt<float>(g, rt, out, st);
}

template <typename T, int NT>
static Error launch_refresh_t(const CacheGeom& g, const RowTable& rt, const void* feat, hipStream_t st) {
  const bool vec = aligned_for_vec<T>(g.base, g.E) && aligned_for_vec<T>(feat, g.E);
  dim3 grid(grid_x_for(g.E, Vec<T>::N * 2), rt.n, g.n_slots);
  if (vec) refresh_kernel<T, NT, true><<<grid, kThreads, 0, st>>>(g, rt, static_cast<const T*>(feat));
  else refresh_kernel<T, NT, false><<<grid, kThreads, 0, st>>>(g, rt, static_cast<const T*>(feat));
  SPECA_HIP(hipGetLastError());
  return ok();
}

template <typename T>
static Error launch_refresh_nt(const CacheGeom& g, const RowTable& rt, const void* feat, hipStream_t st) {
  int mo = 0;
  for (int i = 0; i < rt.n; ++i) mo = rt.order[i] > mo ? rt.order[i] : mo;
  switch (mo) {
    case 0: return launch_refresh_t<T, 1>(g, rt, feat, st);
    case 1: return launch_refresh_t<T, 2>(g, rt, feat, st);
    case 2: return launch_refresh_t<T, 3>(g, rt, feat, st);
    case 3: return launch_refresh_t<T, 4>(g, rt, feat, st);
    default: return launch_refresh_t<T, 5>(g, rt, feat, st);
  }
}

Error launch_refresh(const CacheGeom& g, const RowTable& rt, const void* feat, hipStream_t st) {
  if (rt.n <= 0 || rt.n > kMaxRows) SPECA_FAIL(SPECA_EINVAL, "refresh: %d rows in one launch", rt.n);
  return g.dtype == SPECA_BF16 ? launch_refresh_nt<bf16_t>(g, rt, feat, st) : launch_refresh_nt<float>(g, rt, feat, st);
}

namespace {
typedef unsigned int warm_u32x4 __attribute__((ext_vector_type(4)));
constexpr int kWarmPerThread = 4;
__global__ __launch_bounds__(256) void cache_warm_kernel(CacheGeom g, RowTable rt, int slot, int64_t bytes_per_tensor, int esz) {
  const int i = blockIdx.y / SPECA_MAX_ORDER, o = blockIdx.y % SPECA_MAX_ORDER;
  if (o >= rt.order[i]) return;
  const char* base = static_cast<const char*>(g.base) + g.offset(slot, o, rt.row[i]) * esz;
  const int64_t first = (static_cast<int64_t>(blockIdx.x) * kWarmPerThread * 256 + threadIdx.x) * 16;
  warm_u32x4 acc = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int u = 0; u < kWarmPerThread; ++u) {
    const int64_t off = first + static_cast<int64_t>(u) * 256 * 16;
    if (off + 16 <= bytes_per_tensor) acc ^= *reinterpret_cast<const warm_u32x4*>(base + off);
  }
  asm volatile("" ::"v"(acc));      // the values are not needed, the loads are
}
}  // namespace

Error launch_cache_warm(const CacheGeom& g, const RowTable& rt, int slot, hipStream_t st) {
  if (rt.n <= 0 || rt.n > kMaxRows) SPECA_FAIL(SPECA_EINVAL, "cache warm: %d rows in one launch", rt.n);
  if (slot < 0 || slot >= g.n_slots) SPECA_FAIL(SPECA_EINVAL, "cache warm: slot %d", slot);
  int mo = 0;
  for (int i = 0; i < rt.n; ++i) {
    if (rt.order[i] < 0 || rt.order[i] > g.m) SPECA_FAIL(SPECA_EINVAL, "cache warm: order %d", rt.order[i]);
    mo = rt.order[i] > mo ? rt.order[i] : mo;
  }
  if (mo == 0) return ok();                            // first references: nothing old to read
  const int esz = static_cast<int>(dtype_size(g.dtype));
  const int64_t bytes = g.E * esz;
  if (bytes % 16) return ok();                                // only a hint: skip odd geometries
  dim3 grid(static_cast<unsigned>((bytes + 256 * 16 * kWarmPerThread - 1) / (256 * 16 * kWarmPerThread)), rt.n * SPECA_MAX_ORDER);
  cache_warm_kernel<<<grid, 256, 0, st>>>(g, rt, slot, bytes, esz);
  SPECA_HIP(hipGetLastError());
  return ok();
}

int verify_chunks(int64_t E) { return static_cast<int>((E + kChunk - 1) / kChunk); }

template <typename T, typename TT, int METRIC, bool PC, int NT>
static void launch_verify_partial(const void* pred, const void* truth, int64_t E, const CacheGeom& g, const RowTable& rt,
                                  int slot, int n_rows, float* partial, bool vec, hipStream_t st) {
  dim3 grid(verify_chunks(E), n_rows);
  if (vec)
    verify_partial_kernel<T, TT, METRIC, PC, NT, true><<<grid, kThreads, 0, st>>>(
        static_cast<const T*>(pred), static_cast<const TT*>(truth), E, g, rt, slot, partial, grid.x);
  else
    verify_partial_kernel<T, TT, METRIC, PC, NT, false><<<grid, kThreads, 0, st>>>(
        static_cast<const T*>(pred), static_cast<const TT*>(truth), E, g, rt, slot, partial, grid.x);
}

template <typename T, typename TT, int METRIC>
static void dispatch_verify(const void* pred, const void* truth, int64_t E, const CacheGeom* g, const RowTable* rt, int slot,
                            int n_rows, float* partial, bool vec, hipStream_t st) {
  if (!g) {
    CacheGeom g0{};
    RowTable rt0{};
    launch_verify_partial<T, TT, METRIC, false, 1>(pred, truth, E, g0, rt0, 0, n_rows, partial, vec, st);
    return;
  }
  int mo = 0;
  for (int i = 0; i < rt->n; ++i) mo = rt->order[i] > mo ? rt->order[i] : mo;
  switch (mo) {
    case 0: launch_verify_partial<T, TT, METRIC, true, 1>(nullptr, truth, E, *g, *rt, slot, n_rows, partial, vec, st); break;
    case 1: launch_verify_partial<T, TT, METRIC, true, 2>(nullptr, truth, E, *g, *rt, slot, n_rows, partial, vec, st); break;
    case 2: launch_verify_partial<T, TT, METRIC, true, 3>(nullptr, truth, E, *g, *rt, slot, n_rows, partial, vec, st); break;
    case 3: launch_verify_partial<T, TT, METRIC, true, 4>(nullptr, truth, E, *g, *rt, slot, n_rows, partial, vec, st); break;
    default: launch_verify_partial<T, TT, METRIC, true, 5>(nullptr, truth, E, *g, *rt, slot, n_rows, partial, vec, st); break;
  }
}

template <int METRIC>
static Error launch_verify_m(const void* pred, int pred_dtype, const void* truth, int truth_dtype, int64_t E, const CacheGeom* g,
                             const RowTable* rt, int slot, int n_rows, float eps, const float* tau_dev, float* partial,
                             float* err_dev, uint8_t* accept_dev, hipStream_t st) {
  bool vec = (E % 8 == 0) && (reinterpret_cast<uintptr_t>(truth) % 16 == 0);
  if (g) vec = vec && (reinterpret_cast<uintptr_t>(g->base) % 16 == 0);
  else vec = vec && (reinterpret_cast<uintptr_t>(pred) % 16 == 0);
  const bool pb = pred_dtype == SPECA_BF16, tb = truth_dtype == SPECA_BF16;
  if (pb && tb) dispatch_verify<bf16_t, bf16_t, METRIC>(pred, truth, E, g, rt, slot, n_rows, partial, vec, st);
  else if (pb && !tb) dispatch_verify<bf16_t, float, METRIC>(pred, truth, E, g, rt, slot, n_rows, partial, vec, st);
  else if (!pb && tb) dispatch_verify<float, bf16_t, METRIC>(pred, truth, E, g, rt, slot, n_rows, partial, vec, st);
  else dispatch_verify<float, float, METRIC>(pred, truth, E, g, rt, slot, n_rows, partial, vec, st);
  SPECA_HIP(hipGetLastError());
  verify_final_kernel<METRIC><<<n_rows, 64, 0, st>>>(partial, verify_chunks(E), eps, tau_dev, err_dev, accept_dev);
  SPECA_HIP(hipGetLastError());
  return ok();
}

Error launch_verify(int metric, const void* pred, int pred_dtype, const void* truth, int truth_dtype, int64_t E,
                    const CacheGeom* g, const RowTable* rt, int slot, int n_rows, float eps, const float* tau_dev,
                    float* partial, float* err_dev, uint8_t* accept_dev, hipStream_t st) {
  // the cache form takes its rows from a row table; two tensors can be reduced for more rows at once
  if (n_rows <= 0 || n_rows > (g ? kMaxRows : kMaxVerifyRows)) SPECA_FAIL(SPECA_EINVAL, "verify: %d rows in one launch", n_rows);
  if (E <= 0) SPECA_FAIL(SPECA_EINVAL, "verify: elems_per_row = %lld", static_cast<long long>(E));
  switch (metric) {
    case SPECA_METRIC_L2: return launch_verify_m<SPECA_METRIC_L2>(pred, pred_dtype, truth, truth_dtype, E, g, rt, slot, n_rows, eps, tau_dev, partial, err_dev, accept_dev, st);
    case SPECA_METRIC_L1: return launch_verify_m<SPECA_METRIC_L1>(pred, pred_dtype, truth, truth_dtype, E, g, rt, slot, n_rows, eps, tau_dev, partial, err_dev, accept_dev, st);
    case SPECA_METRIC_LINF: return launch_verify_m<SPECA_METRIC_LINF>(pred, pred_dtype, truth, truth_dtype, E, g, rt, slot, n_rows, eps, tau_dev, partial, err_dev, accept_dev, st);
    case SPECA_METRIC_COSINE: return launch_verify_m<SPECA_METRIC_COSINE>(pred, pred_dtype, truth, truth_dtype, E, g, rt, slot, n_rows, eps, tau_dev, partial, err_dev, accept_dev, st);
  }
  SPECA_FAIL(SPECA_EINVAL, "verify: unknown metric %d", metric);
}

}  // namespace speca
