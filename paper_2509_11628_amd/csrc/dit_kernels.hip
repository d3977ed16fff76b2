// Small kernels of the DiT forward around the contractions: timestep sinusoid,
// conditioning sum, patch embedding, LayerNorm + adaLN modulation, the fused
// forecast-and-fold of speculative steps, un-patchify.
#include "dit_kernels.h"

namespace speca {

namespace {

template <typename T> __device__ inline float ldf(const T* p);
template <> __device__ inline float ldf<float>(const float* p) { return *p; }
template <> __device__ inline float ldf<bf16_t>(const bf16_t* p) { return bf16_to_f32(p->bits); }
template <typename T> __device__ inline void stf(T* p, float v);
template <> __device__ inline void stf<float>(float* p, float v) { *p = v; }
template <> __device__ inline void stf<bf16_t>(bf16_t* p, float v) { p->bits = f32_to_bf16(v); }

// emb[i][j] = cos(t w_j) for j < half, sin(t w_{j-half}) after; w_j = 10000^(-j/half)
template <typename T>
__global__ void sinusoid_kernel(T* __restrict__ emb, int n, int dim, float t) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n * dim) return;
  const int j = idx % dim;
  const int half = dim / 2;
  const int jj = j < half ? j : j - half;
  // fp64 here: the angle reaches ~1e3 rad, where an fp32 frequency would cost 1e-4 of absolute accuracy
  const double w = exp(-log(10000.0) * static_cast<double>(jj) / static_cast<double>(half));
  const double a = static_cast<double>(t) * w;
  stf(emb + idx, static_cast<float>(j < half ? cos(a) : sin(a)));
}

// c = temb + y_table[label];  sc = silu(c) in the model dtype (input of the modulation GEMMs)
template <typename T>
__global__ void cond_sum_kernel(const float* __restrict__ temb, const T* __restrict__ y_table, RowLabels labels, int n, int D,
                                T* __restrict__ sc) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n * D) return;
  const int i = idx / D, d = idx - i * D;
  const float c = temb[idx] + ldf(y_table + static_cast<int64_t>(labels.v[i]) * D + d);
  stf(sc + idx, c / (1.0f + expf(-c)));
}

// h[i][t][d] = sum_k patch(x_row)[t][k] Wp[d][k] + bp[d] + pos[t][d];  k = (c, pi, pj)
template <typename T>
__global__ void patch_embed_kernel(const float* __restrict__ x, RowLabels xrow, const T* __restrict__ Wp, const T* __restrict__ bp,
                                   const T* __restrict__ pos, float* __restrict__ h, int n, int C, int Hh, int Ww, int p, int D) {
  const int gw = Ww / p, gh = Hh / p;
  const int Tn = gh * gw;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= static_cast<int64_t>(n) * Tn * D) return;
  const int d = static_cast<int>(idx % D);
  const int t = static_cast<int>((idx / D) % Tn);
  const int i = static_cast<int>(idx / (static_cast<int64_t>(D) * Tn));
  const int ti = t / gw, tj = t - ti * gw;
  const float* xr = x + static_cast<int64_t>(xrow.v[i]) * C * Hh * Ww;
  const int Kp = C * p * p;
  float acc = 0.0f;
  for (int c = 0; c < C; ++c)
    for (int pi = 0; pi < p; ++pi)
      for (int pj = 0; pj < p; ++pj)
        acc = fmaf(xr[(static_cast<int64_t>(c) * Hh + ti * p + pi) * Ww + tj * p + pj],
                   ldf(Wp + static_cast<int64_t>(d) * Kp + (c * p + pi) * p + pj), acc);
  h[idx] = acc + ldf(bp + d) + ldf(pos + static_cast<int64_t>(t) * D + d);
}

// One wave per token: y = LN(h) * (1 + scale[row]) + shift[row], LN without affine, eps 1e-6.
// Statistics in fp32, two passes over registers.
template <typename T, int PER_LANE>
__global__ __launch_bounds__(256) void ln_modulate_kernel(const float* __restrict__ h, const float* __restrict__ shift,
                                                          const float* __restrict__ scale, const float* __restrict__ shift2,
                                                          const float* __restrict__ scale2, int split_tok, int64_t mod_stride,
                                                          T* __restrict__ y, int64_t n_tokens, int tokens_per_row, int D) {
  const int64_t tok = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (tok >= n_tokens) return;
  const int lane = threadIdx.x & 63;
  const int i = static_cast<int>(tok / tokens_per_row);
  const bool second = static_cast<int>(tok - static_cast<int64_t>(i) * tokens_per_row) >= split_tok;   // tokens from split_tok on use the second set
  const float* hp = h + tok * D;
  float v[PER_LANE];
  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < PER_LANE; ++j) {
    const int d = lane + j * 64;
    v[j] = d < D ? hp[d] : 0.0f;
    s += v[j];
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
  const float mu = s / static_cast<float>(D);
  float q = 0.0f;
#pragma unroll
  for (int j = 0; j < PER_LANE; ++j) {
    const int d = lane + j * 64;
    const float c = d < D ? v[j] - mu : 0.0f;
    q = fmaf(c, c, q);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) q += __shfl_xor(q, off, 64);
  const float rstd = rsqrtf(q / static_cast<float>(D) + 1e-6f);
  const float* sh = (second ? shift2 : shift) + static_cast<int64_t>(i) * mod_stride;
  const float* sc = (second ? scale2 : scale) + static_cast<int64_t>(i) * mod_stride;
  T* yp = y + tok * D;
#pragma unroll
  for (int j = 0; j < PER_LANE; ++j) {
    const int d = lane + j * 64;
    if (d < D) stf(yp + d, (v[j] - mu) * rstd * (1.0f + sc[d]) + sh[d]);
  }
}

// Speculative step: h_out[i][e] = h_in[i][e] + sum_{slot in [s0,s1)} gate_slot[i][d] * sum_o c[i][o] D^o[slot][row_i][e]
// (Eq. 2 for every slot, folded into the residual stream; only the hidden state is written).
// gate of slot j for compact row i: mod[i * mod_stride + gate_off[2j + s] + d], s = 0 for elements below
// split_elem (the text tokens of a two-stream block), 1 from there on.
template <typename T, int NT>
__global__ __launch_bounds__(256) void forecast_fold_kernel(CacheGeom g, RowTable rt, const float* __restrict__ h_in,
                                                            float* __restrict__ h_out, const float* __restrict__ mod,
                                                            int64_t mod_stride, const int32_t* __restrict__ gate_off, int64_t split_elem,
                                                            int s0, int s1, int D) {
  constexpr int V = 4;     // 4 elements per thread: 16 B of fp32 hidden, 8 B (bf16) or 16 B (fp32) of cache
  const int i = blockIdx.y;
  const int64_t e = (static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x) * V;
  if (e >= g.E) return;
  const int d = static_cast<int>(e % D);
  const int row = rt.row[i];
  const int order = rt.order[i];
  float c[NT];
#pragma unroll
  for (int o = 0; o < NT; ++o) c[o] = o <= order ? rt.w[i][o] : 0.0f;
  const T* base = static_cast<const T*>(g.base);
  const float4 hv = *reinterpret_cast<const float4*>(h_in + static_cast<int64_t>(i) * g.E + e);
  float acc[V] = {hv.x, hv.y, hv.z, hv.w};
  const float* mrow = mod + static_cast<int64_t>(i) * mod_stride + d;
  for (int slot = s0; slot < s1; ++slot) {
    const float4 gv = *reinterpret_cast<const float4*>(mrow + gate_off[2 * slot + (e >= split_elem ? 1 : 0)]);
    const float gg[V] = {gv.x, gv.y, gv.z, gv.w};
    float f[V] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int o = 0; o < NT; ++o)
      if (o <= order) {
        float t4[V];
        const T* p = base + g.offset(slot, o, row) + e;
        if (sizeof(T) == 2) {
          const uint2 r = *reinterpret_cast<const uint2*>(p);
          t4[0] = __uint_as_float(r.x << 16); t4[1] = __uint_as_float(r.x & 0xFFFF0000u);
          t4[2] = __uint_as_float(r.y << 16); t4[3] = __uint_as_float(r.y & 0xFFFF0000u);
        } else {
          const float4 r = *reinterpret_cast<const float4*>(p);
          t4[0] = r.x; t4[1] = r.y; t4[2] = r.z; t4[3] = r.w;
        }
#pragma unroll
        for (int q = 0; q < V; ++q) f[q] = fmaf(c[o], t4[q], f[q]);
      }
#pragma unroll
    for (int q = 0; q < V; ++q) acc[q] = fmaf(gg[q], f[q], acc[q]);
  }
  *reinterpret_cast<float4*>(h_out + static_cast<int64_t>(i) * g.E + e) = make_float4(acc[0], acc[1], acc[2], acc[3]);
}

// model_out[row][c][i*p+pi][j*p+pj] = tok[i_compact][t=(i,j)][(c,pi,pj)]
__global__ void unpatchify_kernel(const float* __restrict__ tok, RowLabels rows, float* __restrict__ out, int n, int C, int Hh, int Ww,
                                  int p) {
  const int gw = Ww / p;
  const int64_t per = static_cast<int64_t>(C) * Hh * Ww;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= n * per) return;
  const int i = static_cast<int>(idx / per);
  const int64_t r = idx - i * per;
  const int c = static_cast<int>(r / (Hh * Ww));
  const int y = static_cast<int>((r / Ww) % Hh), xw = static_cast<int>(r % Ww);
  const int ti = y / p, pi = y - ti * p, tj = xw / p, pj = xw - tj * p;
  const int t = ti * gw + tj;
  const int Tn = (Hh / p) * gw;
  const int Kp = C * p * p;
  out[static_cast<int64_t>(rows.v[i]) * per + r] = tok[(static_cast<int64_t>(i) * Tn + t) * Kp + (c * p + pi) * p + pj];
}

inline unsigned blocks_for(int64_t n, int per) { return static_cast<unsigned>((n + per - 1) / per); }

}  // namespace

Error launch_sinusoid(int dtype, void* emb, int n, int dim, float t, hipStream_t st) {
  if (dim % 2) SPECA_FAIL(SPECA_EINVAL, "freq_dim must be even");
  if (dtype == SPECA_BF16) sinusoid_kernel<bf16_t><<<blocks_for(static_cast<int64_t>(n) * dim, 256), 256, 0, st>>>(static_cast<bf16_t*>(emb), n, dim, t);
  else sinusoid_kernel<float><<<blocks_for(static_cast<int64_t>(n) * dim, 256), 256, 0, st>>>(static_cast<float*>(emb), n, dim, t);
  SPECA_HIP(hipGetLastError());
  return ok();
}

Error launch_cond_sum(int dtype, const float* temb, const void* y_table, const RowLabels& labels, int n, int D, void* sc, hipStream_t st) {
  if (dtype == SPECA_BF16)
    cond_sum_kernel<bf16_t><<<blocks_for(static_cast<int64_t>(n) * D, 256), 256, 0, st>>>(temb, static_cast<const bf16_t*>(y_table), labels, n, D, static_cast<bf16_t*>(sc));
  else
    cond_sum_kernel<float><<<blocks_for(static_cast<int64_t>(n) * D, 256), 256, 0, st>>>(temb, static_cast<const float*>(y_table), labels, n, D, static_cast<float*>(sc));
  SPECA_HIP(hipGetLastError());
  return ok();
}

Error launch_patch_embed(int dtype, const float* x, const RowLabels& xrow, const void* Wp, const void* bp, const void* pos, float* h,
                         int n, int C, int Hh, int Ww, int p, int D, hipStream_t st) {
  const int64_t total = static_cast<int64_t>(n) * (Hh / p) * (Ww / p) * D;
  if (dtype == SPECA_BF16)
    patch_embed_kernel<bf16_t><<<blocks_for(total, 256), 256, 0, st>>>(x, xrow, static_cast<const bf16_t*>(Wp), static_cast<const bf16_t*>(bp), static_cast<const bf16_t*>(pos), h, n, C, Hh, Ww, p, D);
  else
    patch_embed_kernel<float><<<blocks_for(total, 256), 256, 0, st>>>(x, xrow, static_cast<const float*>(Wp), static_cast<const float*>(bp), static_cast<const float*>(pos), h, n, C, Hh, Ww, p, D);
  SPECA_HIP(hipGetLastError());
  return ok();
}

template <typename T>
static Error ln_mod_t(const float* h, const float* shift, const float* scale, const float* shift2, const float* scale2, int split_tok,
                      int64_t mod_stride, void* y, int64_t n_tokens, int tokens_per_row, int D, hipStream_t st) {
  const unsigned grid = blocks_for(n_tokens, 4);
  T* yp = static_cast<T*>(y);
  const int per = (D + 63) / 64;
  if (per <= 1) ln_modulate_kernel<T, 1><<<grid, 256, 0, st>>>(h, shift, scale, shift2, scale2, split_tok, mod_stride, yp, n_tokens, tokens_per_row, D);
  else if (per <= 4) ln_modulate_kernel<T, 4><<<grid, 256, 0, st>>>(h, shift, scale, shift2, scale2, split_tok, mod_stride, yp, n_tokens, tokens_per_row, D);
  else if (per <= 18) ln_modulate_kernel<T, 18><<<grid, 256, 0, st>>>(h, shift, scale, shift2, scale2, split_tok, mod_stride, yp, n_tokens, tokens_per_row, D);
  else if (per <= 48) ln_modulate_kernel<T, 48><<<grid, 256, 0, st>>>(h, shift, scale, shift2, scale2, split_tok, mod_stride, yp, n_tokens, tokens_per_row, D);
  else SPECA_FAIL(SPECA_EUNSUPPORTED, "LayerNorm: hidden %d > 3072", D);
  SPECA_HIP(hipGetLastError());
  return ok();
}

Error launch_ln_modulate(int dtype, const float* h, const float* shift, const float* scale, int64_t mod_stride, void* y,
                         int64_t n_tokens, int tokens_per_row, int D, hipStream_t st) {
  return launch_ln_modulate2(dtype, h, shift, scale, shift, scale, tokens_per_row, mod_stride, y, n_tokens, tokens_per_row, D, st);
}

Error launch_ln_modulate2(int dtype, const float* h, const float* shift, const float* scale, const float* shift2, const float* scale2,
                          int split_tok, int64_t mod_stride, void* y, int64_t n_tokens, int tokens_per_row, int D, hipStream_t st) {
  return dtype == SPECA_BF16 ? ln_mod_t<bf16_t>(h, shift, scale, shift2, scale2, split_tok, mod_stride, y, n_tokens, tokens_per_row, D, st)
                             : ln_mod_t<float>(h, shift, scale, shift2, scale2, split_tok, mod_stride, y, n_tokens, tokens_per_row, D, st);
}

template <typename T>
static Error fold_t(const CacheGeom& g, const RowTable& rt, const float* h_in, float* h_out, const float* mod, int64_t mod_stride,
                    const int32_t* gate_off, int64_t split_elem, int s0, int s1, int D, hipStream_t st) {
  int mo = 0;
  for (int i = 0; i < rt.n; ++i) mo = rt.order[i] > mo ? rt.order[i] : mo;
  dim3 grid(blocks_for(g.E, 256 * 4), rt.n);
  switch (mo) {
    case 0: forecast_fold_kernel<T, 1><<<grid, 256, 0, st>>>(g, rt, h_in, h_out, mod, mod_stride, gate_off, split_elem, s0, s1, D); break;
    case 1: forecast_fold_kernel<T, 2><<<grid, 256, 0, st>>>(g, rt, h_in, h_out, mod, mod_stride, gate_off, split_elem, s0, s1, D); break;
    case 2: forecast_fold_kernel<T, 3><<<grid, 256, 0, st>>>(g, rt, h_in, h_out, mod, mod_stride, gate_off, split_elem, s0, s1, D); break;
    case 3: forecast_fold_kernel<T, 4><<<grid, 256, 0, st>>>(g, rt, h_in, h_out, mod, mod_stride, gate_off, split_elem, s0, s1, D); break;
    default: forecast_fold_kernel<T, 5><<<grid, 256, 0, st>>>(g, rt, h_in, h_out, mod, mod_stride, gate_off, split_elem, s0, s1, D); break;
  }
  SPECA_HIP(hipGetLastError());
  return ok();
}

Error launch_forecast_fold(const CacheGeom& g, const RowTable& rt, const float* h_in, float* h_out, const float* mod,
                           int64_t mod_stride, const int32_t* gate_off_dev, int64_t split_elem, int s0, int s1, int D, hipStream_t st) {
  if (rt.n <= 0 || rt.n > kMaxRows) SPECA_FAIL(SPECA_EINVAL, "forecast_fold: %d rows", rt.n);
  if (g.E % 4 || D % 4) SPECA_FAIL(SPECA_EUNSUPPORTED, "forecast_fold needs hidden %% 4 == 0");
  if (s0 < 0 || s1 > g.n_slots || s0 > s1) SPECA_FAIL(SPECA_EINVAL, "forecast_fold: slots [%d,%d)", s0, s1);
  if (split_elem < 0 || split_elem % 4) SPECA_FAIL(SPECA_EINVAL, "forecast_fold: split");
  return g.dtype == SPECA_BF16 ? fold_t<bf16_t>(g, rt, h_in, h_out, mod, mod_stride, gate_off_dev, split_elem, s0, s1, D, st)
                               : fold_t<float>(g, rt, h_in, h_out, mod, mod_stride, gate_off_dev, split_elem, s0, s1, D, st);
}

Error launch_unpatchify(const float* tok, const RowLabels& rows, float* out, int n, int C, int Hh, int Ww, int p, hipStream_t st) {
  unpatchify_kernel<<<blocks_for(static_cast<int64_t>(n) * C * Hh * Ww, 256), 256, 0, st>>>(tok, rows, out, n, C, Hh, Ww, p);
  SPECA_HIP(hipGetLastError());
  return ok();
}

}  // namespace speca
