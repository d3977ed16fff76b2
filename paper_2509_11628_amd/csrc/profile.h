// Optional per-kernel-class timing with HIP events on the context's stream, for roofline
// reports: while a profile is open, launch sites bracket their kernels with an event pair
// and state the algorithmic FLOPs and bytes of the launch.
#pragma once

#include <vector>

#include "common.h"

namespace speca {

struct Profiler {
  struct Rec {
    int cls;
    hipEvent_t a, b;
    double flops, bytes;
  };
  bool on = false;
  bool keep_lanes = false;   // time the laned schedule as it runs instead of serialising it
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;

  hipEvent_t get() {
    if (!pool.empty()) {
      hipEvent_t e = pool.back();
      pool.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
  }
  void begin(int cls, double flops, double bytes, hipStream_t st) {
    if (!on) return;
    Rec r{cls, get(), get(), flops, bytes};
    (void)hipEventRecord(r.a, st);
    recs.push_back(r);
  }
  void end(hipStream_t st) {
    if (!on || recs.empty()) return;
    (void)hipEventRecord(recs.back().b, st);
  }
  ~Profiler() {
    for (auto& r : recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (auto e : pool) (void)hipEventDestroy(e);
  }
};

}  // namespace speca
