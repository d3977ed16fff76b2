// Shared declarations of the SpeCa gfx950 library: error plumbing, storage-type
// helpers, the launch-time row tables and the context object.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdarg>
#include <cstdio>
#include <string>
#include <vector>

#include "../../include/speca.h"

namespace speca {

constexpr int kMaxTensors = SPECA_MAX_ORDER + 1;   // D^0 .. D^m
constexpr int kMaxRows = SPECA_MAX_LAUNCH_ROWS;
constexpr int kMaxLanes = 4;   // concurrent row groups of one step

// ---- storage types -----------------------------------------------------------------
// bf16 values travel as raw 16-bit patterns; arithmetic is always fp32.
struct bf16_t { uint16_t bits; };

__host__ __device__ inline float bf16_to_f32(uint16_t b) {
  union { uint32_t u; float f; } v;
  v.u = static_cast<uint32_t>(b) << 16;
  return v.f;
}
// round to nearest, ties to even (NaN payloads are not preserved; the path never makes NaNs on purpose)
__host__ __device__ inline uint16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } v;
  v.f = f;
  uint32_t u = v.u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

inline size_t dtype_size(int dtype) { return dtype == SPECA_BF16 ? 2 : 4; }

// ---- launch-time tables (passed by value as kernel arguments) ------------------------------
// Row i of a compact launch works on cache row row[i] with its own available order and
// its own fp32 weights: forecast coefficients c_i (Eq. 2) or reciprocal divisors of the
// difference recursion (Eq. 3).  row[i] indexes the [plane][batch_rows] grid of a slot:
// row + plane * batch_rows with planes 0..order[i] counted from there.  The plane part is
// non-zero only for a refresh in the ring layout (order 0: one store into the row's next plane).
struct RowTable {
  int32_t n;
  int32_t row[kMaxRows];
  int32_t order[kMaxRows];
  float w[kMaxRows][kMaxTensors];
};

// Geometry of the cache: [slot][order 0..m][batch_rows][E] elements of the storage type.
struct CacheGeom {
  void* base;
  int64_t E;            // elements per (slot, order, row) = tokens * hidden
  int32_t n_slots;
  int32_t m;            // allocated order
  int32_t batch_rows;
  int32_t dtype;
  __host__ __device__ int64_t offset(int slot, int i, int row) const {
    return ((static_cast<int64_t>(slot) * (m + 1) + i) * batch_rows + row) * E;
  }
};

// ---- errors ----------------------------------------------------------------------------
struct Error {
  int code;
  std::string msg;
};

inline std::string format(const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  return std::string(buf);
}

#define SPECA_FAIL(code_, ...) return ::speca::Error{code_, ::speca::format(__VA_ARGS__)}
#define SPECA_HIP(expr)                                                                     \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return ::speca::Error{SPECA_EHIP, ::speca::format("%s failed: %s", #expr, hipGetErrorString(e_))}; \
  } while (0)
#define SPECA_TRY(expr)                  \
  do {                                   \
    ::speca::Error e__ = (expr);         \
    if (e__.code != SPECA_OK) return e__; \
  } while (0)
inline Error ok() { return Error{SPECA_OK, {}}; }

}  // namespace speca
