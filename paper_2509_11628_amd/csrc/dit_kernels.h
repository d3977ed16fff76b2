// Launchers of the small DiT kernels (see dit_kernels.hip).
#pragma once

#include "common.h"

namespace speca {

// Per-launch integer table passed by value: labels, source rows or destination rows of
// the compact rows of a launch.
struct RowLabels {
  int32_t v[kMaxRows];
};

Error launch_sinusoid(int dtype, void* emb, int n, int dim, float t, hipStream_t st);
Error launch_cond_sum(int dtype, const float* temb, const void* y_table, const RowLabels& labels, int n, int D, void* sc, hipStream_t st);
Error launch_patch_embed(int dtype, const float* x, const RowLabels& xrow, const void* Wp, const void* bp, const void* pos, float* h,
                         int n, int C, int Hh, int Ww, int p, int D, hipStream_t st);
// y = LN(h) * (1 + scale[row]) + shift[row]; shift/scale rows are mod_stride floats apart.
Error launch_ln_modulate(int dtype, const float* h, const float* shift, const float* scale, int64_t mod_stride, void* y,
                         int64_t n_tokens, int tokens_per_row, int D, hipStream_t st);
// Same, tokens [split_tok, tokens_per_row) of every row take (shift2, scale2): the two streams of a dual block.
Error launch_ln_modulate2(int dtype, const float* h, const float* shift, const float* scale, const float* shift2, const float* scale2,
                          int split_tok, int64_t mod_stride, void* y, int64_t n_tokens, int tokens_per_row, int D, hipStream_t st);
// h_out = h_in + sum over slots [s0, s1) of gate * forecast (Eq. 2 fused into the residual stream).
// gate_off_dev: int32[2 * n_slots], entry 2j for elements below split_elem, 2j+1 from there on.
Error launch_forecast_fold(const CacheGeom& g, const RowTable& rt, const float* h_in, float* h_out, const float* mod,
                           int64_t mod_stride, const int32_t* gate_off_dev, int64_t split_elem, int s0, int s1, int D, hipStream_t st);
// One pass for both hidden states of a speculative attempt: h_mid = h_in + slots [s0, s_mid), h_out = h_in + slots [s0, s1);
// s0 <= s_mid < s1 (s_mid == s0: h_mid = h_in).  h_in may be h_mid (in place).
Error launch_forecast_fold2(const CacheGeom& g, const RowTable& rt, const float* h_in, float* h_mid, int s_mid, float* h_out, const float* mod,
                            int64_t mod_stride, const int32_t* gate_off_dev, int64_t split_elem, int s0, int s1, int D, hipStream_t st);
Error launch_unpatchify(const float* tok, const RowLabels& rows, float* out, int n, int C, int Hh, int Ww, int p, hipStream_t st);

}  // namespace speca
