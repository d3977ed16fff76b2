// Host-side schedule logic (see sched.h).  No device code.
#include "sched.h"

#include <cmath>
#include <cstring>
#include <new>

namespace speca {

bool forecast_coefficients(int mode, int step, const int32_t* refs, int n_refs, int order, float* c) {
  if (!refs || !c || n_refs < 1 || order < 0 || order > SPECA_MAX_ORDER || order > n_refs - 1) return false;
  const int k = step - refs[0];
  if (k <= 0) return false;
  if (mode == SPECA_COEF_TAYLOR) {
    double p = 1.0, fact = 1.0;
    for (int i = 0; i <= order; ++i) {
      if (i > 0) { p *= static_cast<double>(k); fact *= static_cast<double>(i); }
      c[i] = static_cast<float>(p / fact);
    }
    return true;
  }
  if (mode == SPECA_COEF_NEWTON) {
    double p = 1.0;
    for (int i = 0; i <= order; ++i) {
      c[i] = static_cast<float>(p);
      p *= static_cast<double>(step - refs[i]);
    }
    return true;
  }
  if (mode == SPECA_COEF_ADAMS_BASHFORTH) {
    // One explicit Adams step of size k in backward-difference form, y + k * sum_j gamma_j nabla^j f,
    // on the slopes between references; the cache holds nabla^j f / g^j as D^{j+1} (g = last gap).
    static const double gamma[SPECA_MAX_ORDER] = {1.0, 1.0 / 2.0, 5.0 / 12.0, 3.0 / 8.0};
    const double g = n_refs >= 2 ? static_cast<double>(refs[0] - refs[1]) : 1.0;
    if (g <= 0.0) return false;
    c[0] = 1.0f;
    double gp = 1.0;
    for (int i = 1; i <= order; ++i) {
      c[i] = static_cast<float>(static_cast<double>(k) * gamma[i - 1] * gp);
      gp *= g;
    }
    return true;
  }
  return false;
}

bool refresh_divisors(int mode, int step, const int32_t* refs, int n_refs, int order, float* d) {
  if (order == 0) return true;
  if (!refs || !d || order < 0 || order > SPECA_MAX_ORDER || n_refs < order) return false;
  for (int i = 1; i <= order; ++i) {
    int div;
    if (mode == SPECA_COEF_TAYLOR || mode == SPECA_COEF_ADAMS_BASHFORTH) div = step - refs[0];
    else if (mode == SPECA_COEF_NEWTON) div = step - refs[i - 1];
    else return false;
    if (div <= 0) return false;
    d[i - 1] = static_cast<float>(div);
  }
  return true;
}

bool RingWeights::push(int mode, int step, const RefHistory& before, int m) {
  if (m < 0 || m > SPECA_MAX_ORDER || (before.n > 0 && step <= before.r[0])) return false;
  const int order = before.n < m ? before.n : m;        // differences defined after this step
  float d[SPECA_MAX_ORDER + 1] = {0};
  if (!refresh_divisors(mode, step, before.r, before.n, order, d)) return false;
  double nw[SPECA_MAX_ORDER + 1][SPECA_MAX_ORDER + 1] = {};
  nw[0][0] = 1.0;
  for (int i = 1; i <= order; ++i)
    for (int j = 0; j <= i; ++j) {
      const double shifted_old = j >= 1 ? W[i - 1][j - 1] : 0.0;
      nw[i][j] = (nw[i - 1][j] - shifted_old) / static_cast<double>(d[i - 1]);
    }
  std::memcpy(W, nw, sizeof(W));
  head = next_plane(m);
  count = count < m + 1 ? count + 1 : m + 1;
  return true;
}

bool RingWeights::forecast(int mode, int step, const RefHistory& h, int m, float* w, int* planes) const {
  if (!w || !planes || head < 0 || count < 1 || h.n < 1) return false;
  const int order = (m < h.n - 1 ? m : h.n - 1) < count - 1 ? (m < h.n - 1 ? m : h.n - 1) : count - 1;
  float c[SPECA_MAX_ORDER + 1] = {0};
  if (!forecast_coefficients(mode, step, h.r, h.n, order, c)) return false;
  for (int p = 0; p < count; ++p) w[p] = 0.0f;
  for (int j = 0; j <= order; ++j) {                      // feature of age j lives `j` planes behind the head
    double acc = 0.0;
    for (int i = j; i <= order; ++i) acc += static_cast<double>(c[i]) * W[i][j];
    w[((head - j) % (m + 1) + (m + 1)) % (m + 1)] = static_cast<float>(acc);
  }
  *planes = count;
  return true;
}

void tau_geometric(float tau0, float beta, int steps, float* out) {
  for (int s = 0; s < steps; ++s)
    out[s] = static_cast<float>(static_cast<double>(tau0) * std::pow(static_cast<double>(beta), static_cast<double>(s) / steps));
}

void tau_linear(float a, float b, int steps, float* out) {
  if (steps == 1) { out[0] = a; return; }
  for (int s = 0; s < steps; ++s)
    out[s] = static_cast<float>(static_cast<double>(a) + (static_cast<double>(b) - static_cast<double>(a)) * (static_cast<double>(s) / (steps - 1)));
}

}  // namespace speca

static bool cfg_valid(const speca_cfg* c) {
  return c && c->order >= 0 && c->order <= SPECA_MAX_ORDER && c->interval >= 1 && c->warmup_full >= 1 &&
         (c->coef_mode == SPECA_COEF_TAYLOR || c->coef_mode == SPECA_COEF_NEWTON || c->coef_mode == SPECA_COEF_ADAMS_BASHFORTH) && c->eps >= 0.0f &&
         c->metric >= SPECA_METRIC_L2 && c->metric <= SPECA_METRIC_COSINE && c->verify_block >= -1 &&
         (c->layout == SPECA_CACHE_DIFFERENCES || c->layout == SPECA_CACHE_RING);
}

extern "C" {

int speca_tau_geometric(float tau0, float beta, int steps, float* tau_out) {
  if (!tau_out || steps < 1 || !(beta > 0.0f)) return SPECA_EINVAL;
  speca::tau_geometric(tau0, beta, steps, tau_out);
  return SPECA_OK;
}

int speca_tau_linear(float tau_start, float tau_end, int steps, float* tau_out) {
  if (!tau_out || steps < 1) return SPECA_EINVAL;
  speca::tau_linear(tau_start, tau_end, steps, tau_out);
  return SPECA_OK;
}

int speca_coefficients(int coef_mode, int step, const int32_t* refs, int n_refs, int order, float* c_out) {
  return speca::forecast_coefficients(coef_mode, step, refs, n_refs, order, c_out) ? SPECA_OK : SPECA_EINVAL;
}

int speca_divisors(int coef_mode, int step, const int32_t* refs, int n_refs, int order, float* d_out) {
  if (order < 0 || (order > 0 && !d_out)) return SPECA_EINVAL;
  return speca::refresh_divisors(coef_mode, step, refs, n_refs, order, d_out) ? SPECA_OK : SPECA_EINVAL;
}

int speca_ring_weights(int coef_mode, int order, const int32_t* full_steps, int n_full, int step, float* w_out, int32_t* plane_out,
                       int* n_out) {
  if (!full_steps || n_full < 1 || !w_out || !plane_out || !n_out || order < 0 || order > SPECA_MAX_ORDER) return SPECA_EINVAL;
  speca::RefHistory h;
  speca::RingWeights ring;
  for (int i = 0; i < n_full; ++i) {
    if (!ring.push(coef_mode, full_steps[i], h, order)) return SPECA_EINVAL;
    h.push(full_steps[i], order);
  }
  float w[SPECA_MAX_ORDER + 1];
  int planes = 0;
  if (!ring.forecast(coef_mode, step, h, order, w, &planes)) return SPECA_EINVAL;
  for (int j = 0; j < planes; ++j) {                       // report by age: 0 = latest feature
    const int p = ((ring.head - j) % (order + 1) + (order + 1)) % (order + 1);
    w_out[j] = w[p];
    plane_out[j] = p;
  }
  *n_out = planes;
  return SPECA_OK;
}

int speca_sched_create(speca_sched** out, int batch, const speca_cfg* cfg) {
  if (!out) return SPECA_EINVAL;
  *out = nullptr;
  if (batch < 1 || !cfg_valid(cfg)) return SPECA_EINVAL;
  speca_sched* s = new (std::nothrow) speca_sched();
  if (!s) return SPECA_ENOMEM;
  s->batch = batch;
  s->cfg = *cfg;
  s->refs.assign(batch, speca::RefHistory());
  *out = s;
  return SPECA_OK;
}

int speca_sched_destroy(speca_sched* s) {
  delete s;
  return SPECA_OK;
}

// A sample speculates at `step` iff it has a reference, fewer than N steps have passed since
// it, the warm-up is over and the threshold is positive; otherwise it is computed in full.
int speca_sched_plan(speca_sched* s, int step, float tau_s, int32_t* spec_out, int* n_spec, int32_t* full_out, int* n_full) {
  if (!s || !spec_out || !n_spec || !full_out || !n_full || step < 0) return SPECA_EINVAL;
  s->planned_spec.clear();
  s->planned_full.clear();
  for (int b = 0; b < s->batch; ++b) {
    const speca::RefHistory& h = s->refs[b];
    if (h.n > 0 && step <= h.r[0]) return SPECA_ESTATE;
    const bool spec = h.n >= 1 && (step - h.r[0]) < s->cfg.interval && step >= s->cfg.warmup_full && tau_s > 0.0f;
    (spec ? s->planned_spec : s->planned_full).push_back(b);
  }
  *n_spec = static_cast<int>(s->planned_spec.size());
  *n_full = static_cast<int>(s->planned_full.size());
  for (int i = 0; i < *n_spec; ++i) spec_out[i] = s->planned_spec[i];
  for (int i = 0; i < *n_full; ++i) full_out[i] = s->planned_full[i];
  s->planned_step = step;
  return SPECA_OK;
}

int speca_sched_commit(speca_sched* s, int step, const uint8_t* accept, int8_t* kind_out) {
  if (!s || step != s->planned_step) return s ? SPECA_ESTATE : SPECA_EINVAL;
  if (!s->planned_spec.empty() && !accept) return SPECA_EINVAL;
  for (size_t i = 0; i < s->planned_spec.size(); ++i) {
    const int b = s->planned_spec[i];
    if (accept[i]) {
      if (kind_out) kind_out[b] = SPECA_KIND_SPEC;          // accepted: cache and references untouched
    } else {
      s->refs[b].push(step, s->cfg.order);                  // rejected: recomputed in full, new reference
      if (kind_out) kind_out[b] = SPECA_KIND_REJECT;
    }
  }
  for (int b : s->planned_full) {
    s->refs[b].push(step, s->cfg.order);
    if (kind_out) kind_out[b] = SPECA_KIND_FULL;
  }
  s->planned_step = -1;
  return SPECA_OK;
}

int speca_sched_refs(const speca_sched* s, int sample, int32_t* refs_out, int* n_out) {
  if (!s || !refs_out || !n_out || sample < 0 || sample >= s->batch) return SPECA_EINVAL;
  const speca::RefHistory& h = s->refs[sample];
  *n_out = h.n;
  for (int i = 0; i < h.n; ++i) refs_out[i] = h.r[i];
  return SPECA_OK;
}

}  // extern "C"
