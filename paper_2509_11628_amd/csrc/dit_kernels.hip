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

// h[i][t][d] = sum_k patch(x_row)[t][k] Wp[d][k] + bp[d] + pos[t][d];  k = (c, pi, pj).
// One thread per (token, 4 consecutive d): the patch values are read once per 4 outputs and are
// wave-uniform loads when D >= 256; the result is stored as one float4.
template <typename T>
__global__ __launch_bounds__(256) void patch_embed_kernel(const float* __restrict__ x, RowLabels xrow, const T* __restrict__ Wp,
                                                          const T* __restrict__ bp, const T* __restrict__ pos, float* __restrict__ h,
                                                          int n, int C, int Hh, int Ww, int p, int D) {
  const int gw = Ww / p, gh = Hh / p;
  const int Tn = gh * gw;
  const int dq = D >> 2;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= static_cast<int64_t>(n) * Tn * dq) return;
  const int d = static_cast<int>(idx % dq) * 4;
  const int t = static_cast<int>((idx / dq) % Tn);
  const int i = static_cast<int>(idx / (static_cast<int64_t>(dq) * Tn));
  const int ti = t / gw, tj = t - ti * gw;
  const float* xr = x + static_cast<int64_t>(xrow.v[i]) * C * Hh * Ww + (static_cast<int64_t>(ti) * p) * Ww + tj * p;
  const int Kp = C * p * p;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (Kp == 16 && p == 2) {
    // the common 2x2 x 4-channel patch: the 16 patch values in registers, weight rows as 16-/32-byte vectors
    float xv[16];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int pi = 0; pi < 2; ++pi) {
        const float2 t2 = *reinterpret_cast<const float2*>(xr + (static_cast<int64_t>(c) * Hh + pi) * Ww);
        xv[(c * 2 + pi) * 2] = t2.x;
        xv[(c * 2 + pi) * 2 + 1] = t2.y;
      }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float w[16];
      const T* wp = Wp + static_cast<int64_t>(d + q) * 16;
      if (sizeof(T) == 2) {
        const uint4 a = *reinterpret_cast<const uint4*>(wp), b = *reinterpret_cast<const uint4*>(wp + 8);
        const uint32_t u[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) { w[2 * j] = __uint_as_float(u[j] << 16); w[2 * j + 1] = __uint_as_float(u[j] & 0xFFFF0000u); }
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float4 a = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(wp) + 4 * j);
          w[4 * j] = a.x; w[4 * j + 1] = a.y; w[4 * j + 2] = a.z; w[4 * j + 3] = a.w;
        }
      }
#pragma unroll
      for (int k = 0; k < 16; ++k) acc[q] = fmaf(xv[k], w[k], acc[q]);
    }
  } else {
    int k = 0;
    for (int c = 0; c < C; ++c)
      for (int pi = 0; pi < p; ++pi)
        for (int pj = 0; pj < p; ++pj, ++k) {
          const float xv = xr[(static_cast<int64_t>(c) * Hh + pi) * Ww + pj];
#pragma unroll
          for (int q = 0; q < 4; ++q) acc[q] = fmaf(xv, ldf(Wp + static_cast<int64_t>(d + q) * Kp + k), acc[q]);
        }
  }
  float r[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) r[q] = acc[q] + ldf(bp + d + q) + ldf(pos + static_cast<int64_t>(t) * D + d + q);
  *reinterpret_cast<float4*>(h + (static_cast<int64_t>(i) * Tn + t) * D + d) = make_float4(r[0], r[1], r[2], r[3]);
}

// One wave per token: y = LN(h) * (1 + scale[row]) + shift[row], LN without affine, eps 1e-6.
// Statistics in fp32, two passes over registers.  Each lane owns quads of four consecutive
// channels (16-byte loads of h, shift and scale, 8- or 16-byte stores of y).
template <typename T, int QUADS>
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
  const int nq = D >> 2;
  float4 v[QUADS];
  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < QUADS; ++j) {
    const int q = lane + j * 64;
    v[j] = q < nq ? *reinterpret_cast<const float4*>(hp + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
    s += (v[j].x + v[j].y) + (v[j].z + v[j].w);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
  const float mu = s / static_cast<float>(D);
  float qs = 0.0f;
#pragma unroll
  for (int j = 0; j < QUADS; ++j) {
    const int q = lane + j * 64;
    if (q < nq) {
      const float a = v[j].x - mu, b = v[j].y - mu, c = v[j].z - mu, d = v[j].w - mu;
      qs += (a * a + b * b) + (c * c + d * d);
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) qs += __shfl_xor(qs, off, 64);
  const float rstd = rsqrtf(qs / static_cast<float>(D) + 1e-6f);
  const float* sh = (second ? shift2 : shift) + static_cast<int64_t>(i) * mod_stride;
  const float* sc = (second ? scale2 : scale) + static_cast<int64_t>(i) * mod_stride;
  T* yp = y + tok * D;
#pragma unroll
  for (int j = 0; j < QUADS; ++j) {
    const int q = lane + j * 64;
    if (q < nq) {
      const float4 a = *reinterpret_cast<const float4*>(sh + 4 * q), b = *reinterpret_cast<const float4*>(sc + 4 * q);
      const float r0 = (v[j].x - mu) * rstd * (1.0f + b.x) + a.x, r1 = (v[j].y - mu) * rstd * (1.0f + b.y) + a.y;
      const float r2 = (v[j].z - mu) * rstd * (1.0f + b.z) + a.z, r3 = (v[j].w - mu) * rstd * (1.0f + b.w) + a.w;
      if (sizeof(T) == 2) {
        uint2 o;
        o.x = static_cast<uint32_t>(f32_to_bf16(r0)) | (static_cast<uint32_t>(f32_to_bf16(r1)) << 16);
        o.y = static_cast<uint32_t>(f32_to_bf16(r2)) | (static_cast<uint32_t>(f32_to_bf16(r3)) << 16);
        *reinterpret_cast<uint2*>(yp + 4 * q) = o;
      } else {
        *reinterpret_cast<float4*>(yp + 4 * q) = make_float4(r0, r1, r2, r3);
      }
    }
  }
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Speculative step: h_out[i][e] = h_in[i][e] + sum_{slot in [s0,s1)} gate_slot[i][d] * sum_o c[i][o] D^o[slot][row_i][e]
// (Eq. 2 for every slot, folded into the residual stream; only the hidden state is written).
// With h_mid != nullptr the running sum after slots [s0, s_mid) is written there as well: the hidden state that
// enters the verify block and the one the accepted path finishes from come out of one pass over the cache.
// gate of slot j for compact row i: mod[i * mod_stride + gate_off[2j + s] + d], s = 0 for elements below
// split_elem (the text tokens of a two-stream block), 1 from there on.
// A thread owns 8 consecutive elements at each of TOK positions half a row apart (TOK = 2 needs an even number of
// tokens: both positions then have the same channel d, and, when no stream boundary falls inside the row, the same
// gate: one gate load serves two sets of cache loads; the gates are 40 % of the load instructions otherwise).
template <typename T, int NT, int TOK, int UNROLL>
__global__ __launch_bounds__(256) void forecast_fold_kernel(CacheGeom g, RowTable rt, const float* h_in,   // h_in may be h_out (in place)
                                                            float* h_out, float* h_mid, int s_mid, const float* __restrict__ mod,
                                                            int64_t mod_stride, const int32_t* __restrict__ gate_off, int64_t split_elem,
                                                            int s0, int s1, int D) {
  constexpr int V = 8;     // 8 elements per position: 2 x 16 B of fp32 hidden, 16 B (bf16) or 2 x 16 B (fp32) of every cached tensor
  const int i = blockIdx.y;
  const int64_t EP = g.E / TOK;                                                // distance of a thread's positions
  const int64_t e = (static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x) * V;
  if (e >= EP) return;
  const int d = static_cast<int>(e % D);
  const int row = rt.row[i];
  const int order = rt.order[i];
  // Orders above this row's available one get coefficient 0 and re-read the highest valid tensor
  // (finite data), so the loads of a slot are unconditional and can all be in flight together.
  float c[NT];
  int oc[NT];
#pragma unroll
  for (int o = 0; o < NT; ++o) {
    c[o] = o <= order ? rt.w[i][o] : 0.0f;
    oc[o] = o <= order ? o : order;
  }
  const T* base = static_cast<const T*>(g.base);
  float acc[TOK][V];
#pragma unroll
  for (int t = 0; t < TOK; ++t) {
    const float* hp = h_in + static_cast<int64_t>(i) * g.E + e + t * EP;
    const float4 h0 = *reinterpret_cast<const float4*>(hp), h1 = *reinterpret_cast<const float4*>(hp + 4);
    acc[t][0] = h0.x; acc[t][1] = h0.y; acc[t][2] = h0.z; acc[t][3] = h0.w;
    acc[t][4] = h1.x; acc[t][5] = h1.y; acc[t][6] = h1.z; acc[t][7] = h1.w;
  }
  const float* mrow = mod + static_cast<int64_t>(i) * mod_stride + d;
  const bool sel = e >= split_elem;                                           // TOK > 1 is only launched when this holds for a whole row
  auto store = [&](float* dst) {
#pragma unroll
    for (int t = 0; t < TOK; ++t) {
      float* p = dst + static_cast<int64_t>(i) * g.E + e + t * EP;
      *reinterpret_cast<float4*>(p) = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
      *reinterpret_cast<float4*>(p + 4) = make_float4(acc[t][4], acc[t][5], acc[t][6], acc[t][7]);
    }
  };
  // TOK * UNROLL * NT cache loads in flight per lane (measured best: 12 with one position, 6 with two)
  auto fold = [&](int sa, int sb) {
#pragma unroll UNROLL
    for (int slot = sa; slot < sb; ++slot) {
      const int off0 = gate_off[2 * slot], off1 = gate_off[2 * slot + 1];     // block-uniform: scalar loads
      const float* gp = mrow + (sel ? off1 : off0);
      const float4 g0 = *reinterpret_cast<const float4*>(gp), g1 = *reinterpret_cast<const float4*>(gp + 4);
      const float gg[V] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
      float t8[TOK][NT][V];
#pragma unroll
      for (int t = 0; t < TOK; ++t)
#pragma unroll
        for (int o = 0; o < NT; ++o) {
          const T* p = base + g.offset(slot, oc[o], row) + e + t * EP;
          if (sizeof(T) == 2) {
            const u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));     // read once per step: keep it out of the caches' way
#pragma unroll
            for (int q = 0; q < 4; ++q) { t8[t][o][2 * q] = __uint_as_float(r[q] << 16); t8[t][o][2 * q + 1] = __uint_as_float(r[q] & 0xFFFF0000u); }
          } else {
            const float4 r0 = *reinterpret_cast<const float4*>(p), r1 = *reinterpret_cast<const float4*>(p + 4);
            t8[t][o][0] = r0.x; t8[t][o][1] = r0.y; t8[t][o][2] = r0.z; t8[t][o][3] = r0.w;
            t8[t][o][4] = r1.x; t8[t][o][5] = r1.y; t8[t][o][6] = r1.z; t8[t][o][7] = r1.w;
          }
        }
#pragma unroll
      for (int t = 0; t < TOK; ++t) {
        float f[V];
#pragma unroll
        for (int q = 0; q < V; ++q) f[q] = 0.0f;
#pragma unroll
        for (int o = 0; o < NT; ++o)
#pragma unroll
          for (int q = 0; q < V; ++q) f[q] = fmaf(c[o], t8[t][o][q], f[q]);
#pragma unroll
        for (int q = 0; q < V; ++q) acc[t][q] = fmaf(gg[q], f[q], acc[t][q]);
      }
    }
  };
  if (h_mid) {                                                                // block-uniform
    fold(s0, s_mid);
    store(h_mid);
    fold(s_mid, s1);
  } else {
    fold(s0, s1);
  }
  store(h_out);
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
  if (D % 4) SPECA_FAIL(SPECA_EUNSUPPORTED, "patch embed: hidden %d is not a multiple of 4", D);
  const int64_t total = static_cast<int64_t>(n) * (Hh / p) * (Ww / p) * (D / 4);
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
  if (D % 4) SPECA_FAIL(SPECA_EUNSUPPORTED, "LayerNorm: hidden %d is not a multiple of 4", D);
  const int per = (D / 4 + 63) / 64;          // quads per lane
  if (per <= 1) ln_modulate_kernel<T, 1><<<grid, 256, 0, st>>>(h, shift, scale, shift2, scale2, split_tok, mod_stride, yp, n_tokens, tokens_per_row, D);
  else if (per <= 2) ln_modulate_kernel<T, 2><<<grid, 256, 0, st>>>(h, shift, scale, shift2, scale2, split_tok, mod_stride, yp, n_tokens, tokens_per_row, D);
  else if (per <= 5) ln_modulate_kernel<T, 5><<<grid, 256, 0, st>>>(h, shift, scale, shift2, scale2, split_tok, mod_stride, yp, n_tokens, tokens_per_row, D);
  else if (per <= 12) ln_modulate_kernel<T, 12><<<grid, 256, 0, st>>>(h, shift, scale, shift2, scale2, split_tok, mod_stride, yp, n_tokens, tokens_per_row, D);
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

template <typename T, int NT>
static Error fold_launch(const CacheGeom& g, const RowTable& rt, const float* h_in, float* h_out, float* h_mid, int s_mid, const float* mod,
                         int64_t mod_stride, const int32_t* gate_off, int64_t split_elem, int s0, int s1, int D, hipStream_t st) {
  // two positions per thread when both see the same channel and the same gate: an even number of tokens, no stream boundary inside the row
  const bool two = g.E % (2 * static_cast<int64_t>(D)) == 0 && (split_elem == 0 || split_elem >= g.E);
  if (two) {
    const dim3 grid(blocks_for(g.E / 2, 256 * 8), rt.n);
    forecast_fold_kernel<T, NT, 2, 1><<<grid, 256, 0, st>>>(g, rt, h_in, h_out, h_mid, s_mid, mod, mod_stride, gate_off, split_elem >= g.E ? g.E : 0, s0, s1, D);
  } else {
    const dim3 grid(blocks_for(g.E, 256 * 8), rt.n);
    forecast_fold_kernel<T, NT, 1, 4><<<grid, 256, 0, st>>>(g, rt, h_in, h_out, h_mid, s_mid, mod, mod_stride, gate_off, split_elem, s0, s1, D);
  }
  SPECA_HIP(hipGetLastError());
  return ok();
}

template <typename T>
static Error fold_t(const CacheGeom& g, const RowTable& rt, const float* h_in, float* h_out, float* h_mid, int s_mid, const float* mod,
                    int64_t mod_stride, const int32_t* gate_off, int64_t split_elem, int s0, int s1, int D, hipStream_t st) {
  int mo = 0;
  for (int i = 0; i < rt.n; ++i) mo = rt.order[i] > mo ? rt.order[i] : mo;
  switch (mo) {
    case 0: return fold_launch<T, 1>(g, rt, h_in, h_out, h_mid, s_mid, mod, mod_stride, gate_off, split_elem, s0, s1, D, st);
    case 1: return fold_launch<T, 2>(g, rt, h_in, h_out, h_mid, s_mid, mod, mod_stride, gate_off, split_elem, s0, s1, D, st);
    case 2: return fold_launch<T, 3>(g, rt, h_in, h_out, h_mid, s_mid, mod, mod_stride, gate_off, split_elem, s0, s1, D, st);
    case 3: return fold_launch<T, 4>(g, rt, h_in, h_out, h_mid, s_mid, mod, mod_stride, gate_off, split_elem, s0, s1, D, st);
    default: return fold_launch<T, 5>(g, rt, h_in, h_out, h_mid, s_mid, mod, mod_stride, gate_off, split_elem, s0, s1, D, st);
  }
}

Error launch_forecast_fold(const CacheGeom& g, const RowTable& rt, const float* h_in, float* h_out, const float* mod,
                           int64_t mod_stride, const int32_t* gate_off_dev, int64_t split_elem, int s0, int s1, int D, hipStream_t st) {
  return launch_forecast_fold2(g, rt, h_in, nullptr, s0, h_out, mod, mod_stride, gate_off_dev, split_elem, s0, s1, D, st);
}

Error launch_forecast_fold2(const CacheGeom& g, const RowTable& rt, const float* h_in, float* h_mid, int s_mid, float* h_out, const float* mod,
                            int64_t mod_stride, const int32_t* gate_off_dev, int64_t split_elem, int s0, int s1, int D, hipStream_t st) {
  if (rt.n <= 0 || rt.n > kMaxRows) SPECA_FAIL(SPECA_EINVAL, "forecast_fold: %d rows", rt.n);
  if (h_mid && (s_mid < s0 || s_mid >= s1)) SPECA_FAIL(SPECA_EINVAL, "forecast_fold: intermediate state after slot %d of [%d,%d)", s_mid, s0, s1);
  if (g.E % 8 || D % 8) SPECA_FAIL(SPECA_EUNSUPPORTED, "forecast_fold needs hidden %% 8 == 0");
  if (s0 < 0 || s1 > g.n_slots || s0 > s1) SPECA_FAIL(SPECA_EINVAL, "forecast_fold: slots [%d,%d)", s0, s1);
  if (split_elem < 0 || split_elem % 8) SPECA_FAIL(SPECA_EINVAL, "forecast_fold: split");
  return g.dtype == SPECA_BF16 ? fold_t<bf16_t>(g, rt, h_in, h_out, h_mid, s_mid, mod, mod_stride, gate_off_dev, split_elem, s0, s1, D, st)
                               : fold_t<float>(g, rt, h_in, h_out, h_mid, s_mid, mod, mod_stride, gate_off_dev, split_elem, s0, s1, D, st);
}

Error launch_unpatchify(const float* tok, const RowLabels& rows, float* out, int n, int C, int Hh, int Ww, int p, hipStream_t st) {
  unpatchify_kernel<<<blocks_for(static_cast<int64_t>(n) * C * Hh * Ww, 256), 256, 0, st>>>(tok, rows, out, n, C, Hh, Ww, p);
  SPECA_HIP(hipGetLastError());
  return ok();
}

}  // namespace speca
