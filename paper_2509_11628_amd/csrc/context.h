// The library context: cache, per-row reference histories, verification scratch and
// (optionally) a target model.
#pragma once

#include <memory>
#include <string>
#include <vector>

#include "common.h"
#include "profile.h"
#include "sched.h"

namespace speca {

struct Model;

// Small pinned host area + device mirrors for the per-launch scalars that travel each
// speculative step (thresholds in; errors and verdicts out).
struct VerifyScratch {
  float* tau_dev = nullptr;        // [kMaxRows]
  float* err_dev = nullptr;        // [kMaxRows]
  uint8_t* acc_dev = nullptr;      // [kMaxRows]
  float* partial = nullptr;        // [rows][chunks][3]
  size_t partial_cap = 0;          // floats
  float* h_tau = nullptr;          // pinned [kMaxRows]
  float* h_err = nullptr;          // pinned [kMaxRows]
  uint8_t* h_acc = nullptr;        // pinned [kMaxRows]
};

}  // namespace speca

struct speca_ctx {
  speca_model_desc desc{};
  hipStream_t stream = nullptr;
  int device = 0;
  std::string err;

  bool cache_ready = false;
  speca_cfg cfg{};
  int batch_rows = 0;
  speca::CacheGeom geom{};
  size_t cache_cap = 0;                       // bytes allocated at geom.base
  std::vector<speca::RefHistory> row_refs;    // per cache row

  speca::VerifyScratch vs;
  std::unique_ptr<speca::Model> model;
  speca::Profiler prof;

  int64_t elems_per_slot_row() const { return geom.E; }
};

namespace speca {

// Brackets the launches made in its scope with an event pair when a profile is open.
struct ProfScope {
  speca_ctx* c;
  ProfScope(speca_ctx* ctx, int cls, double flops, double bytes) : c(ctx) { c->prof.begin(cls, flops, bytes, c->stream); }
  ~ProfScope() { c->prof.end(c->stream); }
};
inline double table_tensors(const RowTable& rt) {   // sum over rows of (order + 1)
  double t = 0;
  for (int i = 0; i < rt.n; ++i) t += rt.order[i] + 1;
  return t;
}

// Fill a RowTable with forecast coefficients for rows[0..n) at `step` (Eq. 2).
Error build_forecast_table(const speca_ctx* ctx, int step, const int32_t* rows, int n, RowTable* rt);
// Fill a RowTable with reciprocal divisors for a refresh of rows[0..n) at `step` (Eq. 3 recursion).
Error build_refresh_table(const speca_ctx* ctx, int step, const int32_t* rows, int n, RowTable* rt);
// Record `step` as the latest reference of the rows.
void push_refs(speca_ctx* ctx, int step, const int32_t* rows, int n);
Error ensure_partial(speca_ctx* ctx, size_t floats);
Error check_rows(const speca_ctx* ctx, const int32_t* rows, int n_rows);

}  // namespace speca
