// Drives the host-only part of the C ABI (schedule state machine, forecast coefficients, refresh divisors, ring
// weights, threshold helpers) through seeded random sequences and through its error paths.  Built by
// tests/test_host_sanitizers.py together with csrc/sched.cpp under AddressSanitizer and UndefinedBehaviorSanitizer:
// any out-of-bounds access, use after free, leak or undefined operation aborts the run.  Values are checked
// against the oracle elsewhere (tests/test_host_logic.py); here only structural invariants are asserted.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/speca.h"

#define REQUIRE(cond)                                                     \
  do {                                                                    \
    if (!(cond)) {                                                        \
      std::fprintf(stderr, "%s:%d: %s failed\n", __FILE__, __LINE__, #cond); \
      std::exit(1);                                                       \
    }                                                                     \
  } while (0)

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd() {          // splitmix64
  uint64_t z = (state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return static_cast<uint32_t>((z ^ (z >> 31)) >> 16);
}

int main() {
  // threshold helpers: edge sizes and rejected arguments
  for (int steps : {1, 2, 3, 50, 1000}) {
    std::vector<float> t(steps);
    REQUIRE(speca_tau_geometric(0.1f, 0.2f, steps, t.data()) == SPECA_OK);
    REQUIRE(t[0] == 0.1f);
    REQUIRE(speca_tau_linear(0.05f, 0.01f, steps, t.data()) == SPECA_OK);
    REQUIRE(t[0] == 0.05f);
  }
  float one = 0.f;
  REQUIRE(speca_tau_geometric(0.1f, 0.2f, 0, &one) == SPECA_EINVAL);
  REQUIRE(speca_tau_geometric(0.1f, 0.0f, 4, &one) == SPECA_EINVAL);
  REQUIRE(speca_tau_geometric(0.1f, 0.2f, 4, nullptr) == SPECA_EINVAL);
  REQUIRE(speca_tau_linear(0.1f, 0.2f, -3, &one) == SPECA_EINVAL);

  // coefficients, divisors and ring weights over random irregular histories, every policy and order
  for (int it = 0; it < 4000; ++it) {
    const int mode = static_cast<int>(rnd() % 3);
    const int order = static_cast<int>(rnd() % (SPECA_MAX_ORDER + 1));
    const int n_full = 1 + static_cast<int>(rnd() % 9);
    std::vector<int32_t> full(n_full);
    int s = static_cast<int>(rnd() % 5);
    for (int i = 0; i < n_full; ++i) { full[i] = s; s += 1 + static_cast<int>(rnd() % 6); }
    const int step = full.back() + 1 + static_cast<int>(rnd() % 7);
    // exact-size output buffers: a write past the request is caught
    const int held = n_full < order + 1 ? n_full : order + 1;
    std::vector<int32_t> refs(held);
    for (int i = 0; i < held; ++i) refs[i] = full[n_full - 1 - i];
    const int o = held - 1;
    std::vector<float> c(o + 1), d(o > 0 ? o : 1), w(order + 1);
    std::vector<int32_t> planes(order + 1);
    REQUIRE(speca_coefficients(mode, step, refs.data(), held, o, c.data()) == SPECA_OK);
    REQUIRE(c[0] == 1.0f);
    REQUIRE(speca_divisors(mode, step, refs.data(), held, o, d.data()) == SPECA_OK);
    int n = -1;
    REQUIRE(speca_ring_weights(mode, order, full.data(), n_full, step, w.data(), planes.data(), &n) == SPECA_OK);
    REQUIRE(n == held);
    for (int j = 0; j < n; ++j) REQUIRE(planes[j] >= 0 && planes[j] <= order);
    // invalid requests are refused, not executed
    REQUIRE(speca_coefficients(mode, refs[0], refs.data(), held, o, c.data()) == SPECA_EINVAL);          // step not after the reference
    REQUIRE(speca_coefficients(mode, step, refs.data(), held, held, c.data()) == SPECA_EINVAL);          // order beyond the history
    REQUIRE(speca_coefficients(7, step, refs.data(), held, o, c.data()) == SPECA_EINVAL);
    REQUIRE(speca_coefficients(mode, step, nullptr, held, o, c.data()) == SPECA_EINVAL);
    REQUIRE(speca_ring_weights(mode, SPECA_MAX_ORDER + 1, full.data(), n_full, step, w.data(), planes.data(), &n) == SPECA_EINVAL);
    REQUIRE(speca_ring_weights(mode, order, full.data(), n_full, full.back(), w.data(), planes.data(), &n) == SPECA_EINVAL);
    if (o > 0) REQUIRE(speca_divisors(mode, refs[0], refs.data(), held, o, d.data()) == SPECA_EINVAL);
  }

  // the state machine: random verdicts, every configuration corner
  for (int it = 0; it < 600; ++it) {
    speca_cfg cfg{};
    cfg.order = static_cast<int>(rnd() % (SPECA_MAX_ORDER + 1));
    cfg.interval = 1 + static_cast<int>(rnd() % 7);
    cfg.verify_block = -1;
    cfg.coef_mode = static_cast<int>(rnd() % 3);
    cfg.eps = 1e-8f;
    cfg.warmup_full = 1 + static_cast<int>(rnd() % 3);
    cfg.metric = static_cast<int>(rnd() % 4);
    cfg.layout = static_cast<int>(rnd() % 2);
    const int batch = 1 + static_cast<int>(rnd() % 9);
    speca_sched* sc = nullptr;
    REQUIRE(speca_sched_create(&sc, batch, &cfg) == SPECA_OK && sc);
    std::vector<int32_t> spec(batch), full(batch), refs(SPECA_MAX_ORDER + 1);
    std::vector<uint8_t> acc(batch);
    std::vector<int8_t> kinds(batch);
    std::vector<int> last(batch, -1);
    const int S = 5 + static_cast<int>(rnd() % 40);
    for (int step = 0; step < S; ++step) {
      const float tau = (rnd() % 5 == 0) ? 0.0f : 0.1f;
      int ns = -1, nf = -1;
      REQUIRE(speca_sched_plan(sc, step, tau, spec.data(), &ns, full.data(), &nf) == SPECA_OK);
      REQUIRE(ns >= 0 && nf >= 0 && ns + nf == batch);
      if (tau <= 0.0f || step < cfg.warmup_full) REQUIRE(ns == 0);
      for (int i = 0; i < ns; ++i) {
        REQUIRE(last[spec[i]] >= 0 && step - last[spec[i]] < cfg.interval);
        acc[i] = rnd() % 3 != 0;
      }
      REQUIRE(speca_sched_commit(sc, step + 1, acc.data(), kinds.data()) == SPECA_ESTATE);      // not the planned step
      REQUIRE(speca_sched_commit(sc, step, ns ? acc.data() : nullptr, kinds.data()) == SPECA_OK);
      REQUIRE(speca_sched_commit(sc, step, acc.data(), kinds.data()) == SPECA_ESTATE);          // already committed
      for (int i = 0; i < ns; ++i) {
        REQUIRE(kinds[spec[i]] == (acc[i] ? SPECA_KIND_SPEC : SPECA_KIND_REJECT));
        if (!acc[i]) last[spec[i]] = step;
      }
      for (int i = 0; i < nf; ++i) { REQUIRE(kinds[full[i]] == SPECA_KIND_FULL); last[full[i]] = step; }
      for (int b = 0; b < batch; ++b) {
        int n = -1;
        REQUIRE(speca_sched_refs(sc, b, refs.data(), &n) == SPECA_OK);
        REQUIRE(n >= 1 && n <= cfg.order + 1 && refs[0] == last[b]);
        for (int i = 1; i < n; ++i) REQUIRE(refs[i] < refs[i - 1]);
      }
    }
    int n = 0;
    REQUIRE(speca_sched_refs(sc, batch, refs.data(), &n) == SPECA_EINVAL);
    REQUIRE(speca_sched_refs(sc, -1, refs.data(), &n) == SPECA_EINVAL);
    int ns = 0, nf = 0;
    REQUIRE(speca_sched_plan(sc, 0, 0.1f, spec.data(), &ns, full.data(), &nf) == SPECA_ESTATE);  // a step that is already behind
    REQUIRE(speca_sched_plan(sc, S, 0.1f, nullptr, &ns, full.data(), &nf) == SPECA_EINVAL);
    REQUIRE(speca_sched_destroy(sc) == SPECA_OK);
  }
  // refused configurations allocate nothing that could leak
  speca_cfg bad{};
  bad.order = SPECA_MAX_ORDER + 1; bad.interval = 1; bad.warmup_full = 1;
  speca_sched* none = reinterpret_cast<speca_sched*>(0x1);
  REQUIRE(speca_sched_create(&none, 4, &bad) == SPECA_EINVAL && none == nullptr);
  REQUIRE(speca_sched_create(nullptr, 4, &bad) == SPECA_EINVAL);
  REQUIRE(speca_sched_destroy(nullptr) == SPECA_OK);
  std::puts("host logic: sanitizer run clean");
  return 0;
}
