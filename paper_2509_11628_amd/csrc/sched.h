// Host-side schedule logic of the SpeCa sampler: reference histories, forecast
// coefficients, difference divisors, threshold schedules and the per-sample
// full / speculative state machine (Sec. 3.3, Eq. 2-3; Sec. 3.4.2).
// Pure C++: no device code, testable without a GPU.
#pragma once

#include <stdint.h>

#include <vector>

#include "../../include/speca.h"

namespace speca {

// Steps at which one row (or sample) was computed in full, latest first; at most m+1 kept.
struct RefHistory {
  int32_t n = 0;
  int32_t r[SPECA_MAX_ORDER + 1] = {0, 0, 0, 0, 0};
  void push(int step, int m) {
    int keep = n < m + 1 ? n : m;      // entries that survive
    for (int i = keep; i > 0; --i) r[i] = r[i - 1];
    r[0] = step;
    n = keep + 1;
  }
  void clear() { n = 0; }
};

// Weights c_0..c_order of the cached differences when forecasting `step`.
// TAYLOR (Eq. 2 as printed, differences pre-divided by the gap): c_i = k^i / i!, k = step - refs[0].
// NEWTON (backward divided differences): c_i = prod_{j<i} (step - refs[j]).
// Returns false on an invalid request (no reference, step not after it, order too high).
bool forecast_coefficients(int mode, int step, const int32_t* refs, int n_refs, int order, float* c);

// Divisors d_1..d_order of the recursion D^i <- (D^{i-1}_new - D^{i-1}_old) / d_i at a new
// full step.  TAYLOR: the last gap for every i.  NEWTON: step - refs[i-1].
bool refresh_divisors(int mode, int step, const int32_t* refs, int n_refs, int order, float* d);

// Raw-feature ring layout of the cache: the m+1 planes of a slot hold the features of the last
// m+1 full steps instead of the differences, so a refresh is one store and reads nothing.  The
// differences of Eq. 3 are linear in those features; this keeps, per cache row, the matrix
// W[i][j] with  D^i = sum_j W[i][j] * F(age j)  (age 0 = latest), advanced at every refresh by
// the same recursion the difference layout applies to the tensors:
//   W'[0] = e_0,   W'[i] = (W'[i-1] - shift(W[i-1])) / d_i    (shift: every feature is one older).
// A forecast is then sum_j (sum_i c_i W[i][j]) F(age j): the forecast kernels run unchanged on
// per-plane weights.
struct RingWeights {
  int32_t head = -1;            // plane of the latest feature; -1 = empty
  int32_t count = 0;            // features held, at most m+1
  double W[SPECA_MAX_ORDER + 1][SPECA_MAX_ORDER + 1] = {};
  void clear() { *this = RingWeights(); }
  int next_plane(int m) const { return head < 0 ? 0 : (head + 1) % (m + 1); }
  // Advance for a full step at `step`; `before` is the row's history before that step.
  bool push(int mode, int step, const RefHistory& before, int m);
  // Per-plane weights of the forecast for `step` (history `h` = the row's current one):
  // w[p] for planes p < count, *planes = count.  False on an invalid request.
  bool forecast(int mode, int step, const RefHistory& h, int m, float* w, int* planes) const;
};

void tau_geometric(float tau0, float beta, int steps, float* out);
void tau_linear(float a, float b, int steps, float* out);

}  // namespace speca

// The state machine behind speca_sched_* and speca_sample.
struct speca_sched {
  int batch = 0;
  speca_cfg cfg{};
  std::vector<speca::RefHistory> refs;     // per sample
  std::vector<int32_t> planned_spec, planned_full;
  int planned_step = -1;
};
