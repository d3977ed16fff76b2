// Launchers of the small MMDiT kernels (see mmdit_kernels.hip).
#pragma once

#include "common.h"
#include "dit_kernels.h"

namespace speca {

// In place on a packed qkv buffer [n_tokens][ld] (q at column 0, k at column D = H*hd):
// per head RMS-norm (eps 1e-6) with learned scale, then rotation of the pairs (2i, 2i+1) by the
// token's angle (cos/sin tables [tokens_per_row][hd/2], fp32).  Tokens below split_tok of every
// row take the first scale pair (text stream), the others the second.
Error launch_qk_norm_rope(int dtype, void* qkv, int64_t ld, int64_t n_tokens, int tokens_per_row, int split_tok, int H, int hd,
                          const void* qn1, const void* kn1, const void* qn2, const void* kn2, const float* cos_t, const float* sin_t,
                          hipStream_t st);
// sc = silu(a + b) in the model dtype; a, b fp32 [n][D].
Error launch_silu_sum(int dtype, const float* a, const float* b, void* sc, int64_t n, hipStream_t st);
// Gather rows of a [rows_all][width] matrix (model dtype): dst[i] = src[idx[i]].
Error launch_gather_rows(int dtype, const void* src, const RowLabels& idx, void* dst, int n, int64_t width, hipStream_t st);
// patches[i][t][(c,pi,pj)] in the model dtype from fp32 latents x[row][C][F][H][W]; token t = (f, i, j).
Error launch_patchify(int dtype, const float* x, const RowLabels& xrow, void* patches, int n, int C, int F, int Hh, int Ww, int p,
                      hipStream_t st);
// model_out[row][c][f][i*p+pi][j*p+pj] = tok[i_compact][t][(c,pi,pj)]
Error launch_unpatchify_video(const float* tok, const RowLabels& rows, float* out, int n, int C, int F, int Hh, int Ww, int p,
                              hipStream_t st);

}  // namespace speca
