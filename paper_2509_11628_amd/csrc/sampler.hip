// speca_sample: the whole forecast-then-verify trajectory (Sec. 3.2 workflow, Sec. 3.4.2
// sequential validation) driven from the host, plus the solver update kernel.
#include <algorithm>
#include <cmath>
#include <limits>

#include "context.h"
#include "kernels.h"
#include "model.h"

namespace speca {

namespace {

// DDIM (eta = 0):  x0 = (x - sqrt(1-a) e)/sqrt(a);  x' = sqrt(a') x0 + sqrt(1-a') e
// flow Euler:      x' = x + (sigma' - sigma) v
// DDPM (Eq. 1):    al = a/a', be = 1 - al;  x' = (x - be/sqrt(1-a) e)/sqrt(al) + sqrt(be) z  (z = nullptr: the mean)
// Guidance:        e = e_u + scale (e_c - e_u), conditional rows first, unconditional rows after.
__global__ __launch_bounds__(256) void solver_update_kernel(int kind, float* __restrict__ x, const float* __restrict__ out,
                                                            int64_t total, int64_t uncond_offset, float cfg_scale, float ta,
                                                            float tb, const float* __restrict__ z) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= total) return;
  float e = out[i];
  if (cfg_scale > 0.0f) {
    const float eu = out[i + uncond_offset];
    e = eu + cfg_scale * (e - eu);
  }
  const float xv = x[i];
  float r;
  if (kind == SPECA_SOLVER_DDIM) {
    const float x0 = (xv - sqrtf(1.0f - ta) * e) / sqrtf(ta);
    r = sqrtf(tb) * x0 + sqrtf(1.0f - tb) * e;
  } else if (kind == SPECA_SOLVER_FLOW) {
    r = xv + (tb - ta) * e;
  } else {
    const float al = ta / tb, be = 1.0f - al;
    r = (xv - be / sqrtf(1.0f - ta) * e) / sqrtf(al);
    if (z) r += sqrtf(be) * z[i];
  }
  x[i] = r;
}

}  // namespace

Error launch_solver_update(int kind, float* latents, const float* model_out, int batch, int64_t n, float cfg_scale, float tab_s,
                           float tab_next, const float* draws, hipStream_t st) {
  const int64_t total = static_cast<int64_t>(batch) * n;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7FFFFFFF) SPECA_FAIL(SPECA_EINVAL, "latent too large for one launch");
  solver_update_kernel<<<static_cast<unsigned>(blocks), 256, 0, st>>>(kind, latents, model_out, total, total, cfg_scale, tab_s,
                                                                     tab_next, draws);
  SPECA_HIP(hipGetLastError());
  return ok();
}

Error sample_impl(speca_ctx* ctx, float* latents, int batch, const speca_cond* cond, const speca_solver* solver, const float* tau,
                  speca_trace* trace) {
  if (!ctx->model) SPECA_FAIL(SPECA_EUNSUPPORTED, "this context has no model (cache-only)");
  if (!ctx->cache_ready) SPECA_FAIL(SPECA_ESTATE, "speca_init_cache has not been called");
  if (!latents || !cond || !solver || !tau) SPECA_FAIL(SPECA_EINVAL, "latents, cond, solver and tau must not be NULL");
  if (solver->kind != SPECA_SOLVER_DDIM && solver->kind != SPECA_SOLVER_FLOW && solver->kind != SPECA_SOLVER_DDPM)
    SPECA_FAIL(SPECA_EINVAL, "solver kind = %d", solver->kind);
  if (solver->kind == SPECA_SOLVER_DDPM && !solver->noise) SPECA_FAIL(SPECA_EINVAL, "the DDPM solver needs solver->noise");
  if (solver->steps < 1 || !solver->timesteps || !solver->table) SPECA_FAIL(SPECA_EINVAL, "solver tables missing");
  if (batch < 1) SPECA_FAIL(SPECA_EINVAL, "batch = %d", batch);
  const bool guided = solver->cfg_scale > 0.0f;
  const int R = guided ? 2 : 1;
  if (ctx->batch_rows != R * batch)
    SPECA_FAIL(SPECA_ESTATE, "cache was initialised for %d rows, this call needs %d", ctx->batch_rows, R * batch);
  const int S = solver->steps;
  const int B = batch;

  // per-row labels: conditional rows carry the sample's label, unconditional rows the null label
  std::vector<int32_t> labels(ctx->batch_rows, 0);
  if (ctx->desc.kind == SPECA_MODEL_DIT) {
    if (!cond->labels) SPECA_FAIL(SPECA_EINVAL, "cond->labels is NULL");
    for (int b = 0; b < B; ++b) {
      if (cond->labels[b] < 0 || cond->labels[b] > ctx->desc.num_classes) SPECA_FAIL(SPECA_EINVAL, "label of sample %d out of range", b);
      labels[b] = cond->labels[b];
      if (guided) labels[B + b] = ctx->desc.num_classes;
    }
  }

  // fresh trajectory: forget all references
  clear_refs(ctx);
  speca_sched sched;
  sched.batch = B;
  sched.cfg = ctx->cfg;
  sched.refs.assign(B, RefHistory());

  const int64_t n = ctx->model->latent_elems();
  float* model_out = ctx->model_out;           // [batch_rows][n], sized by speca_init_cache
  if (!model_out) SPECA_FAIL(SPECA_ESTATE, "the model-output workspace is missing");

  std::vector<int32_t> spec(B), full(B), rows;
  std::vector<uint8_t> accept(B);
  std::vector<int8_t> kinds(B);
  std::vector<float> tau_rows(kMaxRows);
  if (trace) trace->n_full = trace->n_spec = trace->n_reject = 0;
  const float nan = std::numeric_limits<float>::quiet_NaN();
  const int samples_per_launch = kMaxRows / R;

  SPECA_TRY(ctx->model->begin_trajectory(ctx, cond, labels.data(), solver->timesteps, S));
  struct TrajGuard { Model* m; ~TrajGuard() { m->end_trajectory(); } } traj_guard{ctx->model.get()};

  for (int s = 0; s < S; ++s) {
    speca_cond c = *cond;
    c.timestep = solver->timesteps[s];
    int n_spec = 0, n_full = 0;
    if (speca_sched_plan(&sched, s, tau[s], spec.data(), &n_spec, full.data(), &n_full) != SPECA_OK)
      SPECA_FAIL(SPECA_ESTATE, "scheduler rejected step %d", s);
    if (trace && trace->err)
      for (int b = 0; b < B; ++b) trace->err[(static_cast<int64_t>(b) * S + s) * 2] = trace->err[(static_cast<int64_t>(b) * S + s) * 2 + 1] = nan;

    for (int i0 = 0; i0 < n_spec; i0 += samples_per_launch) {
      const int ns = std::min(samples_per_launch, n_spec - i0);
      rows.clear();
      for (int i = 0; i < ns; ++i) rows.push_back(spec[i0 + i]);
      if (guided)
        for (int i = 0; i < ns; ++i) rows.push_back(B + spec[i0 + i]);
      for (size_t i = 0; i < rows.size(); ++i) tau_rows[i] = tau[s];
      SPECA_TRY(ctx->model->spec_step(ctx, latents, B, &c, labels.data(), s, rows.data(), static_cast<int>(rows.size()),
                                      tau_rows.data(), guided ? B : 0, model_out));
      for (int i = 0; i < ns; ++i) {
        accept[i0 + i] = ctx->vs.h_acc[i];      // already combined over the pair
        if (trace && trace->err) {
          float* e = trace->err + (static_cast<int64_t>(spec[i0 + i]) * S + s) * 2;
          e[0] = ctx->vs.h_err[i];
          if (guided) e[1] = ctx->vs.h_err[ns + i];
        }
      }
    }
    if (speca_sched_commit(&sched, s, accept.data(), kinds.data()) != SPECA_OK) SPECA_FAIL(SPECA_ESTATE, "scheduler commit failed at step %d", s);

    // rejected samples join the scheduled-full ones: same step, complete forward
    std::vector<int32_t> todo(full.begin(), full.begin() + n_full);
    for (int i = 0; i < n_spec; ++i)
      if (!accept[i]) todo.push_back(spec[i]);
    std::sort(todo.begin(), todo.end());
    for (size_t i0 = 0; i0 < todo.size(); i0 += samples_per_launch) {
      const size_t ns = std::min<size_t>(samples_per_launch, todo.size() - i0);
      rows.clear();
      for (size_t i = 0; i < ns; ++i) rows.push_back(todo[i0 + i]);
      if (guided)
        for (size_t i = 0; i < ns; ++i) rows.push_back(B + todo[i0 + i]);
      SPECA_TRY(ctx->model->full_step(ctx, latents, B, &c, labels.data(), s, rows.data(), static_cast<int>(rows.size()), model_out));
    }
    const float* draws = solver->kind == SPECA_SOLVER_DDPM && s + 1 < S ? solver->noise + static_cast<int64_t>(s) * B * n : nullptr;
    ProfScope ps(ctx, SPECA_PROF_OTHER, 0.0, static_cast<double>(B) * n * 4 * (2 + R + (draws ? 1 : 0)));
    SPECA_TRY(launch_solver_update(solver->kind, latents, model_out, B, n, guided ? solver->cfg_scale : 0.0f, solver->table[s],
                                   solver->table[s + 1], draws, ctx->stream));
    if (trace) {
      for (int b = 0; b < B; ++b) {
        if (trace->kind) trace->kind[static_cast<int64_t>(b) * S + s] = kinds[b];
        if (kinds[b] == SPECA_KIND_SPEC) trace->n_spec++;
        else trace->n_full++;
        if (kinds[b] == SPECA_KIND_REJECT) trace->n_reject++;
      }
    }
  }
  SPECA_HIP(hipStreamSynchronize(ctx->stream));
  return ok();
}

}  // namespace speca
