// Small kernels of the MMDiT forward around the contractions: per-head RMS-norm + rotary
// embedding of q and k, conditioning sum, patchify / un-patchify of (video) latents.
#include "mmdit_kernels.h"

namespace speca {

namespace {

template <typename T> __device__ inline float ldf(const T* p);
template <> __device__ inline float ldf<float>(const float* p) { return *p; }
template <> __device__ inline float ldf<bf16_t>(const bf16_t* p) { return bf16_to_f32(p->bits); }
template <typename T> __device__ inline void stf(T* p, float v);
template <> __device__ inline void stf<float>(float* p, float v) { *p = v; }
template <> __device__ inline void stf<bf16_t>(bf16_t* p, float v) { p->bits = f32_to_bf16(v); }

// two consecutive elements at an even element offset
__device__ inline void ld_pair(const float* p, float& a, float& b) { const float2 v = *reinterpret_cast<const float2*>(p); a = v.x; b = v.y; }
__device__ inline void ld_pair(const bf16_t* p, float& a, float& b) {
  const uint32_t v = *reinterpret_cast<const uint32_t*>(p);
  a = __uint_as_float(v << 16); b = __uint_as_float(v & 0xFFFF0000u);
}
__device__ inline void st_pair(float* p, float a, float b) { *reinterpret_cast<float2*>(p) = make_float2(a, b); }
__device__ inline void st_pair(bf16_t* p, float a, float b) {
  *reinterpret_cast<uint32_t*>(p) = static_cast<uint32_t>(f32_to_bf16(a)) | (static_cast<uint32_t>(f32_to_bf16(b)) << 16);
}

// One wave per (token, group of HG heads); lane i owns the rotation pair (2i, 2i+1) of q and of k of each head.
// The HG heads are independent chains (load, reduce, scale, rotate, store): taking several per wave keeps that
// many loads in flight instead of one round trip at a time.
constexpr int kHeadGroup = 4;
template <typename T>
__global__ __launch_bounds__(256) void qk_norm_rope_kernel(T* __restrict__ qkv, int64_t ld, int64_t n_items, int tokens_per_row,
                                                           int split_tok, int H, int hd, const T* __restrict__ qn1,
                                                           const T* __restrict__ kn1, const T* __restrict__ qn2,
                                                           const T* __restrict__ kn2, const float* __restrict__ cos_t,
                                                           const float* __restrict__ sin_t) {
  constexpr int HG = kHeadGroup;
  const int64_t item = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (item >= n_items) return;
  const int lane = threadIdx.x & 63;
  const int groups = (H + HG - 1) / HG;
  const int64_t tok = item / groups;
  const int head0 = static_cast<int>(item - tok * groups) * HG;
  const int t = static_cast<int>(tok % tokens_per_row);
  const bool second = t >= split_tok;
  const int half = hd / 2;
  const bool live = lane < half;
  T* q[HG];
  float q0[HG], q1[HG], k0[HG], k1[HG];
#pragma unroll
  for (int g = 0; g < HG; ++g) {
    const int head = head0 + g < H ? head0 + g : H - 1;        // a surplus head of the last group re-reads the last head; never stored
    q[g] = qkv + tok * ld + static_cast<int64_t>(head) * hd + 2 * lane;
    q0[g] = q1[g] = k0[g] = k1[g] = 0.0f;
    if (live) { ld_pair(q[g], q0[g], q1[g]); ld_pair(q[g] + static_cast<int64_t>(H) * hd, k0[g], k1[g]); }
  }
  const T* qn = second ? qn2 : qn1;
  const T* kn = second ? kn2 : kn1;
  float nq0 = 0, nq1 = 0, nk0 = 0, nk1 = 0, c = 0, s = 0;
  if (live) {
    ld_pair(qn + 2 * lane, nq0, nq1);
    ld_pair(kn + 2 * lane, nk0, nk1);
    c = cos_t[static_cast<int64_t>(t) * half + lane];
    s = sin_t[static_cast<int64_t>(t) * half + lane];
  }
  float sq[HG], sk[HG];
#pragma unroll
  for (int g = 0; g < HG; ++g) { sq[g] = q0[g] * q0[g] + q1[g] * q1[g]; sk[g] = k0[g] * k0[g] + k1[g] * k1[g]; }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1)
#pragma unroll
    for (int g = 0; g < HG; ++g) { sq[g] += __shfl_xor(sq[g], off, 64); sk[g] += __shfl_xor(sk[g], off, 64); }
  if (!live) return;
#pragma unroll
  for (int g = 0; g < HG; ++g) {
    if (head0 + g >= H) break;
    const float rq = rsqrtf(sq[g] / static_cast<float>(hd) + 1e-6f), rk = rsqrtf(sk[g] / static_cast<float>(hd) + 1e-6f);
    const float a0 = q0[g] * (rq * nq0), a1 = q1[g] * (rq * nq1);
    const float b0 = k0[g] * (rk * nk0), b1 = k1[g] * (rk * nk1);
    st_pair(q[g], a0 * c - a1 * s, a0 * s + a1 * c);
    st_pair(q[g] + static_cast<int64_t>(H) * hd, b0 * c - b1 * s, b0 * s + b1 * c);
  }
}

template <typename T>
__global__ void silu_sum_kernel(const float* __restrict__ a, const float* __restrict__ b, T* __restrict__ sc, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float c = a[i] + b[i];
  stf(sc + i, c / (1.0f + expf(-c)));
}

template <typename T>
__global__ void gather_rows_kernel(const T* __restrict__ src, RowLabels idx, T* __restrict__ dst, int n, int64_t width) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= n * width) return;
  const int r = static_cast<int>(i / width);
  dst[i] = src[static_cast<int64_t>(idx.v[r]) * width + (i - r * width)];
}

template <typename T>
__global__ void patchify_kernel(const float* __restrict__ x, RowLabels xrow, T* __restrict__ patches, int n, int C, int F, int Hh,
                                int Ww, int p) {
  const int gh = Hh / p, gw = Ww / p;
  const int Kp = C * p * p;
  const int64_t Tn = static_cast<int64_t>(F) * gh * gw;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= n * Tn * Kp) return;
  const int kk = static_cast<int>(idx % Kp);
  const int64_t t = (idx / Kp) % Tn;
  const int i = static_cast<int>(idx / (Kp * Tn));
  const int c = kk / (p * p), pi = (kk / p) % p, pj = kk % p;
  const int f = static_cast<int>(t / (gh * gw)), ti = static_cast<int>((t / gw) % gh), tj = static_cast<int>(t % gw);
  const float v = x[(((static_cast<int64_t>(xrow.v[i]) * C + c) * F + f) * Hh + ti * p + pi) * Ww + tj * p + pj];
  stf(patches + idx, v);
}

__global__ void unpatchify_video_kernel(const float* __restrict__ tok, RowLabels rows, float* __restrict__ out, int n, int C, int F,
                                        int Hh, int Ww, int p) {
  const int gh = Hh / p, gw = Ww / p;
  const int64_t per = static_cast<int64_t>(C) * F * Hh * Ww;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= n * per) return;
  const int i = static_cast<int>(idx / per);
  const int64_t r = idx - i * per;
  const int xw = static_cast<int>(r % Ww), y = static_cast<int>((r / Ww) % Hh);
  const int f = static_cast<int>((r / (static_cast<int64_t>(Ww) * Hh)) % F), c = static_cast<int>(r / (static_cast<int64_t>(Ww) * Hh * F));
  const int ti = y / p, pi = y - ti * p, tj = xw / p, pj = xw - tj * p;
  const int64_t t = (static_cast<int64_t>(f) * gh + ti) * gw + tj;
  const int Kp = C * p * p;
  out[static_cast<int64_t>(rows.v[i]) * per + r] = tok[(static_cast<int64_t>(i) * F * gh * gw + t) * Kp + (c * p + pi) * p + pj];
}

inline unsigned nblk(int64_t n, int per) { return static_cast<unsigned>((n + per - 1) / per); }

}  // namespace

Error launch_qk_norm_rope(int dtype, void* qkv, int64_t ld, int64_t n_tokens, int tokens_per_row, int split_tok, int H, int hd,
                          const void* qn1, const void* kn1, const void* qn2, const void* kn2, const float* cos_t, const float* sin_t,
                          hipStream_t st) {
  if (hd % 2 || hd > 128 || hd < 2) SPECA_FAIL(SPECA_EUNSUPPORTED, "qk_norm_rope: head_dim %d", hd);
  // the kernel moves rotation pairs as one 4- / 8-byte access
  const uintptr_t al = reinterpret_cast<uintptr_t>(qkv) | reinterpret_cast<uintptr_t>(qn1) | reinterpret_cast<uintptr_t>(kn1) |
                       reinterpret_cast<uintptr_t>(qn2) | reinterpret_cast<uintptr_t>(kn2);
  if (ld % 2 || al % 8) SPECA_FAIL(SPECA_EUNSUPPORTED, "qk_norm_rope: operands must be 8-byte aligned with an even leading dimension");
  const int64_t items = n_tokens * ((H + kHeadGroup - 1) / kHeadGroup);
  if (items > 4LL * 0x7FFFFFFF) SPECA_FAIL(SPECA_EINVAL, "qk_norm_rope: too many items");
  if (dtype == SPECA_BF16)
    qk_norm_rope_kernel<bf16_t><<<nblk(items, 4), 256, 0, st>>>(static_cast<bf16_t*>(qkv), ld, items, tokens_per_row, split_tok, H, hd,
                                                              static_cast<const bf16_t*>(qn1), static_cast<const bf16_t*>(kn1),
                                                              static_cast<const bf16_t*>(qn2), static_cast<const bf16_t*>(kn2), cos_t, sin_t);
  else
    qk_norm_rope_kernel<float><<<nblk(items, 4), 256, 0, st>>>(static_cast<float*>(qkv), ld, items, tokens_per_row, split_tok, H, hd,
                                                             static_cast<const float*>(qn1), static_cast<const float*>(kn1),
                                                             static_cast<const float*>(qn2), static_cast<const float*>(kn2), cos_t, sin_t);
  SPECA_HIP(hipGetLastError());
  return ok();
}

Error launch_silu_sum(int dtype, const float* a, const float* b, void* sc, int64_t n, hipStream_t st) {
  if (dtype == SPECA_BF16) silu_sum_kernel<bf16_t><<<nblk(n, 256), 256, 0, st>>>(a, b, static_cast<bf16_t*>(sc), n);
  else silu_sum_kernel<float><<<nblk(n, 256), 256, 0, st>>>(a, b, static_cast<float*>(sc), n);
  SPECA_HIP(hipGetLastError());
  return ok();
}

Error launch_gather_rows(int dtype, const void* src, const RowLabels& idx, void* dst, int n, int64_t width, hipStream_t st) {
  if (dtype == SPECA_BF16)
    gather_rows_kernel<uint16_t><<<nblk(n * width, 256), 256, 0, st>>>(static_cast<const uint16_t*>(src), idx, static_cast<uint16_t*>(dst), n, width);
  else
    gather_rows_kernel<float><<<nblk(n * width, 256), 256, 0, st>>>(static_cast<const float*>(src), idx, static_cast<float*>(dst), n, width);
  SPECA_HIP(hipGetLastError());
  return ok();
}

Error launch_patchify(int dtype, const float* x, const RowLabels& xrow, void* patches, int n, int C, int F, int Hh, int Ww, int p,
                      hipStream_t st) {
  const int64_t total = static_cast<int64_t>(n) * F * (Hh / p) * (Ww / p) * C * p * p;
  if (dtype == SPECA_BF16) patchify_kernel<bf16_t><<<nblk(total, 256), 256, 0, st>>>(x, xrow, static_cast<bf16_t*>(patches), n, C, F, Hh, Ww, p);
  else patchify_kernel<float><<<nblk(total, 256), 256, 0, st>>>(x, xrow, static_cast<float*>(patches), n, C, F, Hh, Ww, p);
  SPECA_HIP(hipGetLastError());
  return ok();
}

Error launch_unpatchify_video(const float* tok, const RowLabels& rows, float* out, int n, int C, int F, int Hh, int Ww, int p,
                              hipStream_t st) {
  unpatchify_video_kernel<<<nblk(static_cast<int64_t>(n) * C * F * Hh * Ww, 256), 256, 0, st>>>(tok, rows, out, n, C, F, Hh, Ww, p);
  SPECA_HIP(hipGetLastError());
  return ok();
}

}  // namespace speca
