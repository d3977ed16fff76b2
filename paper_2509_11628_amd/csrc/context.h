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
  float* tau_dev = nullptr;        // [kMaxVerifyRows]
  float* err_dev = nullptr;        // [kMaxVerifyRows]
  uint8_t* acc_dev = nullptr;      // [kMaxVerifyRows]
  float* partial = nullptr;        // [rows][chunks][3]
  size_t partial_cap = 0;          // floats
  float* h_tau = nullptr;          // pinned [kMaxVerifyRows]
  float* h_err = nullptr;          // pinned [kMaxVerifyRows]
  uint8_t* h_acc = nullptr;        // pinned [kMaxVerifyRows]
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
  std::vector<speca::RingWeights> row_ring;   // per cache row (ring layout only)

  // Lanes: the rows of one launch are independent, so a step can run its row groups side by side
  // on streams of its own (lane 0 is `stream`).  While one group sits in an HBM-bound epilogue or
  // LayerNorm the other keeps the matrix cores busy, and two half-size GEMMs together fill the CUs
  // that one tile-quantised launch leaves idle.  Fork / join with events; results do not change.
  int lanes = 4;
  hipStream_t lane_stream[speca::kMaxLanes] = {};   // [0] = stream; others library-owned
  hipEvent_t lane_fork = nullptr;
  hipEvent_t lane_join[speca::kMaxLanes] = {};

  speca::VerifyScratch vs;
  float* static_partial = nullptr;            // device address of the file-scope reduction scratch on this context's device
  float* model_out = nullptr;                 // [batch_rows][latent elems] fp32: model outputs of a trajectory's current step
  size_t model_out_cap = 0;                   // bytes
  std::unique_ptr<speca::Model> model;
  speca::Profiler prof;

  int64_t elems_per_slot_row() const { return geom.E; }
};

namespace speca {

// Brackets the launches made in its scope with an event pair when a profile is open.
struct ProfScope {
  speca_ctx* c;
  hipStream_t st;
  ProfScope(speca_ctx* ctx, int cls, double flops, double bytes) : c(ctx), st(ctx->stream) { c->prof.begin(cls, flops, bytes, st); }
  ProfScope(speca_ctx* ctx, hipStream_t stream, int cls, double flops, double bytes) : c(ctx), st(stream) { c->prof.begin(cls, flops, bytes, st); }
  ~ProfScope() { c->prof.end(st); }
};

// Row groups of one launch: lane k takes compact rows [first[k], first[k+1]).
struct LaneSplit {
  int n_lanes = 1;
  int first[kMaxLanes + 1] = {};
};
// Split n rows over the context's lanes (at least min_rows per lane; one lane while a profile is open
// unless the caller asked for lanes explicitly: per-kernel event times are only clean when serial).
LaneSplit split_lanes(const speca_ctx* ctx, int n, int min_rows);
// main stream -> all lanes of the split (they wait for everything enqueued on the main stream so far)
Error lanes_fork(speca_ctx* ctx, const LaneSplit& ls);
// all lanes -> main stream
Error lanes_join(speca_ctx* ctx, const LaneSplit& ls);
// Rows [first, first + n) of a table, as a table of its own.
RowTable slice_table(const RowTable& rt, int first, int n);
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
// Forget every reference (a new trajectory).
void clear_refs(speca_ctx* ctx);
Error ensure_partial(speca_ctx* ctx, size_t floats);
Error check_rows(const speca_ctx* ctx, const int32_t* rows, int n_rows);

}  // namespace speca
