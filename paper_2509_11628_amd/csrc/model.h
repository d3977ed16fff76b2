// Interface between the sampler / C ABI and a target model (DiT, MMDiT).
#pragma once

#include "common.h"
#include "context.h"

namespace speca {

struct Model {
  virtual ~Model() {}
  virtual int n_slots() const = 0;
  virtual int n_blocks() const = 0;
  virtual int64_t tokens() const = 0;           // tokens per row in a cached slot
  virtual int hidden() const = 0;
  virtual int64_t latent_elems() const = 0;     // elements of one row of x / model_out
  // Size workspaces for launches of up to batch_rows rows.
  virtual Error prepare(speca_ctx* ctx, int batch_rows) = 0;
  // Reference step (Sec. 3.2 step 1): full forward of rows[0..n) with the cache refresh fused
  // in.  x row of cache row r is x + (r % x_mod) * latent_elems(); labels are per cache row.
  virtual Error full_step(speca_ctx* ctx, const float* x, int x_mod, const speca_cond* cond, const int32_t* labels_per_row,
                          int step, const int32_t* rows, int n, float* model_out) = 0;
  // Speculative attempt (Sec. 3.2 steps 2-3).  Leaves errors/verdicts in ctx->vs.h_err / h_acc
  // (entry i for rows[i]) after synchronising; accepted rows are finished into model_out.
  virtual Error spec_step(speca_ctx* ctx, const float* x, int x_mod, const speca_cond* cond, const int32_t* labels_per_row,
                          int step, const int32_t* rows, int n, const float* tau_per_row, int pair_stride,
                          float* model_out) = 0;
  // Whole-trajectory preparation: the conditioning of every step is known up front (the solver
  // tables are data), so the modulation of all steps and rows can be one large GEMM instead of a
  // weight-bound skinny one per step.  Optional; steps outside a trajectory compute it themselves.
  virtual Error begin_trajectory(speca_ctx*, const speca_cond*, const int32_t* /*labels_per_row*/, const float* /*timesteps*/, int /*S*/) {
    return ok();
  }
  virtual void end_trajectory() {}
};

// Factories; return nullptr + error on failure.
Error make_dit_model(const speca_model_desc& d, const speca_weights* w, std::unique_ptr<Model>* out);
Error make_mmdit_model(const speca_model_desc& d, const speca_weights* w, std::unique_ptr<Model>* out);

// Solver update on device (DDIM eta=0 or flow Euler) with optional guidance combine.
// latents [batch][n] fp32; model_out [rows][n] fp32, rows = batch or 2*batch.
Error launch_solver_update(int kind, float* latents, const float* model_out, int batch, int64_t n, float cfg_scale,
                           float tab_s, float tab_next, const float* draws, hipStream_t st);

}  // namespace speca
