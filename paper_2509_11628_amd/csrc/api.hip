// C ABI entry points (see include/speca.h): argument validation, cache ownership,
// per-row reference bookkeeping; all arithmetic is in the kernels.
#include <cmath>
#include <cstring>
#include <new>

#include "context.h"
#include "gemm.h"
#include "kernels.h"
#include "model.h"

using namespace speca;

static thread_local std::string g_create_error;

// ---- reduction scratch of the entry point that allocates nothing -------------------------------------------
// speca_verify_static keeps the stage-1 partial sums of Eq. 4 in this file-scope device array instead of a
// hipMalloc'ed buffer.  Every GPU the library runs on holds its own copy at its own address; the name below is
// only a host-side handle: host code uses the device address that hipGetSymbolAddress returned for the
// current device (kept per device in g_static_partial), never the name itself.
constexpr size_t kStaticPartialFloats = SPECA_VERIFY_STATIC_MAX_PARTIALS * 3;      // 768 KiB
static __device__ __align__(256) float scratch[kStaticPartialFloats];
constexpr int kMaxDevices = 64;
static float* g_static_partial[kMaxDevices] = {};

// Device address of the array on `device`, which must be the current device.
static Error static_partial_for(int device, float** out) {
  if (device < 0 || device >= kMaxDevices) SPECA_FAIL(SPECA_EUNSUPPORTED, "device ordinal %d", device);
  if (!g_static_partial[device]) {
    float* p = nullptr;
    SPECA_HIP(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
    if (!p) SPECA_FAIL(SPECA_EHIP, "hipGetSymbolAddress returned a null address");
    g_static_partial[device] = p;
  }
  *out = g_static_partial[device];
  return ok();
}

static int finish(speca_ctx* ctx, const Error& e) {
  if (e.code != SPECA_OK && ctx) ctx->err = e.msg;
  return e.code;
}

namespace speca {

Error check_rows(const speca_ctx* ctx, const int32_t* rows, int n_rows) {
  if (!rows) SPECA_FAIL(SPECA_EINVAL, "rows is NULL");
  if (n_rows <= 0 || n_rows > ctx->batch_rows) SPECA_FAIL(SPECA_EINVAL, "n_rows = %d (cache has %d rows)", n_rows, ctx->batch_rows);
  for (int i = 0; i < n_rows; ++i) {
    if (rows[i] < 0 || rows[i] >= ctx->batch_rows) SPECA_FAIL(SPECA_EINVAL, "rows[%d] = %d out of range", i, rows[i]);
    if (i > 0 && rows[i] <= rows[i - 1]) SPECA_FAIL(SPECA_EINVAL, "rows must be strictly increasing (rows[%d] = %d)", i, rows[i]);
  }
  return ok();
}

Error build_forecast_table(const speca_ctx* ctx, int step, const int32_t* rows, int n, RowTable* rt) {
  if (n > kMaxRows) SPECA_FAIL(SPECA_EINVAL, "more than %d rows in one launch", kMaxRows);
  rt->n = n;
  for (int i = 0; i < n; ++i) {
    const RefHistory& h = ctx->row_refs[rows[i]];
    if (h.n < 1) SPECA_FAIL(SPECA_ESTATE, "row %d has no reference step yet", rows[i]);
    if (step <= h.r[0]) SPECA_FAIL(SPECA_ESTATE, "step %d is not after row %d's latest reference %d", step, rows[i], h.r[0]);
    const int order = std::min(ctx->cfg.order, h.n - 1);
    rt->row[i] = rows[i];
    rt->order[i] = order;
    for (int o = 0; o < kMaxTensors; ++o) rt->w[i][o] = 0.0f;
    if (ctx->cfg.layout == SPECA_CACHE_RING) {
      int planes = 0;                                     // weights per plane; every held plane is read
      if (!ctx->row_ring[rows[i]].forecast(ctx->cfg.coef_mode, step, h, ctx->cfg.order, rt->w[i], &planes))
        SPECA_FAIL(SPECA_EINVAL, "cannot form forecast weights for row %d", rows[i]);
      rt->order[i] = planes - 1;
    } else if (!forecast_coefficients(ctx->cfg.coef_mode, step, h.r, h.n, order, rt->w[i])) {
      SPECA_FAIL(SPECA_EINVAL, "cannot form forecast coefficients for row %d", rows[i]);
    }
  }
  return ok();
}

Error build_refresh_table(const speca_ctx* ctx, int step, const int32_t* rows, int n, RowTable* rt) {
  if (n > kMaxRows) SPECA_FAIL(SPECA_EINVAL, "more than %d rows in one launch", kMaxRows);
  rt->n = n;
  for (int i = 0; i < n; ++i) {
    const RefHistory& h = ctx->row_refs[rows[i]];
    if (h.n > 0 && step <= h.r[0]) SPECA_FAIL(SPECA_ESTATE, "step %d is not after row %d's latest reference %d", step, rows[i], h.r[0]);
    const int order = std::min(ctx->cfg.order, h.n);      // order available after this refresh
    rt->row[i] = rows[i];
    rt->order[i] = order;
    float d[kMaxTensors] = {0};
    for (int o = 0; o < kMaxTensors; ++o) rt->w[i][o] = 0.0f;
    if (ctx->cfg.layout == SPECA_CACHE_RING) {            // one store into the next plane, nothing read
      rt->row[i] = rows[i] + ctx->row_ring[rows[i]].next_plane(ctx->cfg.order) * ctx->batch_rows;
      rt->order[i] = 0;
      continue;
    }
    if (!refresh_divisors(ctx->cfg.coef_mode, step, h.r, h.n, order, d))
      SPECA_FAIL(SPECA_EINVAL, "cannot form refresh divisors for row %d", rows[i]);
    for (int o = 0; o < order; ++o) rt->w[i][o] = 1.0f / d[o];
  }
  return ok();
}

void push_refs(speca_ctx* ctx, int step, const int32_t* rows, int n) {
  for (int i = 0; i < n; ++i) {
    if (ctx->cfg.layout == SPECA_CACHE_RING)
      (void)ctx->row_ring[rows[i]].push(ctx->cfg.coef_mode, step, ctx->row_refs[rows[i]], ctx->cfg.order);   // validated by build_refresh_table
    ctx->row_refs[rows[i]].push(step, ctx->cfg.order);
  }
}

void clear_refs(speca_ctx* ctx) {
  ctx->row_refs.assign(ctx->batch_rows, RefHistory());
  ctx->row_ring.assign(ctx->batch_rows, RingWeights());
}

Error ensure_partial(speca_ctx* ctx, size_t floats) {
  if (ctx->vs.partial_cap >= floats) return ok();
  if (ctx->vs.partial) {
    SPECA_HIP(hipStreamSynchronize(ctx->stream));
    SPECA_HIP(hipFree(ctx->vs.partial));
    ctx->vs.partial = nullptr;
    ctx->vs.partial_cap = 0;
  }
  if (hipMalloc(&ctx->vs.partial, floats * sizeof(float)) != hipSuccess) {
    (void)hipGetLastError();
    SPECA_FAIL(SPECA_ENOMEM, "cannot allocate %zu bytes of reduction scratch", floats * sizeof(float));
  }
  ctx->vs.partial_cap = floats;
  return ok();
}

}  // namespace speca

static bool cfg_ok(const speca_cfg* c, std::string* why) {
  if (!c) { *why = "cfg is NULL"; return false; }
  if (c->order < 0 || c->order > SPECA_MAX_ORDER) { *why = format("order = %d (0..%d)", c->order, SPECA_MAX_ORDER); return false; }
  if (c->interval < 1) { *why = format("interval = %d (>= 1)", c->interval); return false; }
  if (c->warmup_full < 1) { *why = format("warmup_full = %d (>= 1)", c->warmup_full); return false; }
  if (c->coef_mode != SPECA_COEF_TAYLOR && c->coef_mode != SPECA_COEF_NEWTON && c->coef_mode != SPECA_COEF_ADAMS_BASHFORTH) { *why = format("coef_mode = %d", c->coef_mode); return false; }
  if (!(c->eps >= 0.0f)) { *why = "eps < 0"; return false; }
  if (c->metric < SPECA_METRIC_L2 || c->metric > SPECA_METRIC_COSINE) { *why = format("metric = %d", c->metric); return false; }
  if (c->verify_block < -1) { *why = format("verify_block = %d", c->verify_block); return false; }
  if (c->layout != SPECA_CACHE_DIFFERENCES && c->layout != SPECA_CACHE_RING) { *why = format("layout = %d", c->layout); return false; }
  return true;
}

static void free_ctx(speca_ctx* ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);
  for (int k = 1; k < kMaxLanes; ++k)
    if (ctx->lane_stream[k]) { (void)hipStreamSynchronize(ctx->lane_stream[k]); (void)hipStreamDestroy(ctx->lane_stream[k]); }
  if (ctx->lane_fork) (void)hipEventDestroy(ctx->lane_fork);
  for (int k = 0; k < kMaxLanes; ++k)
    if (ctx->lane_join[k]) (void)hipEventDestroy(ctx->lane_join[k]);
  ctx->model.reset();
  if (ctx->geom.base) (void)hipFree(ctx->geom.base);
  if (ctx->model_out) (void)hipFree(ctx->model_out);
  VerifyScratch& v = ctx->vs;
  if (v.tau_dev) (void)hipFree(v.tau_dev);
  if (v.err_dev) (void)hipFree(v.err_dev);
  if (v.acc_dev) (void)hipFree(v.acc_dev);
  if (v.partial) (void)hipFree(v.partial);
  if (v.h_tau) (void)hipHostFree(v.h_tau);
  if (v.h_err) (void)hipHostFree(v.h_err);
  if (v.h_acc) (void)hipHostFree(v.h_acc);
  delete ctx;
}

static Error create_impl(speca_ctx** out, const speca_model_desc* desc, const speca_weights* w, void* hip_stream) {
  if (!desc) SPECA_FAIL(SPECA_EINVAL, "desc is NULL");
  if (desc->dtype != SPECA_F32 && desc->dtype != SPECA_BF16) SPECA_FAIL(SPECA_EINVAL, "dtype = %d", desc->dtype);
  if (desc->hidden < 1) SPECA_FAIL(SPECA_EINVAL, "hidden = %d", desc->hidden);
  std::unique_ptr<speca_ctx, void (*)(speca_ctx*)> ctx(new (std::nothrow) speca_ctx(), free_ctx);
  if (!ctx) SPECA_FAIL(SPECA_ENOMEM, "out of host memory");
  ctx->desc = *desc;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  switch (desc->kind) {
    case SPECA_MODEL_NONE:
      if (desc->n_slots < 1 || desc->tokens < 1) SPECA_FAIL(SPECA_EINVAL, "cache-only context needs n_slots >= 1 and tokens >= 1");
      break;
    case SPECA_MODEL_DIT:
      SPECA_TRY(make_dit_model(*desc, w, &ctx->model));
      break;
    case SPECA_MODEL_MMDIT:
      SPECA_TRY(make_mmdit_model(*desc, w, &ctx->model));
      break;
    default:
      SPECA_FAIL(SPECA_EINVAL, "model kind = %d", desc->kind);
  }
  SPECA_HIP(hipGetDevice(&ctx->device));
  SPECA_TRY(static_partial_for(ctx->device, &ctx->static_partial));      // set-up: the device is current here
  // lane streams: default priority, not synchronising with the NULL stream; ordering is by events only
  ctx->lane_stream[0] = ctx->stream;
  for (int k = 1; k < kMaxLanes; ++k) SPECA_HIP(hipStreamCreateWithFlags(&ctx->lane_stream[k], hipStreamNonBlocking));
  SPECA_HIP(hipEventCreateWithFlags(&ctx->lane_fork, hipEventDisableTiming));
  for (int k = 0; k < kMaxLanes; ++k) SPECA_HIP(hipEventCreateWithFlags(&ctx->lane_join[k], hipEventDisableTiming));
  if (const char* e = getenv("SPECA_LANES")) {
    const int v = atoi(e);
    if (v >= 1 && v <= kMaxLanes) ctx->lanes = v;
  }
  VerifyScratch& v = ctx->vs;
  SPECA_HIP(hipMalloc(&v.tau_dev, kMaxVerifyRows * sizeof(float)));
  SPECA_HIP(hipMalloc(&v.err_dev, kMaxVerifyRows * sizeof(float)));
  SPECA_HIP(hipMalloc(&v.acc_dev, kMaxVerifyRows));
  SPECA_HIP(hipHostMalloc(&v.h_tau, kMaxVerifyRows * sizeof(float), hipHostMallocDefault));
  SPECA_HIP(hipHostMalloc(&v.h_err, kMaxVerifyRows * sizeof(float), hipHostMallocDefault));
  SPECA_HIP(hipHostMalloc(&v.h_acc, kMaxVerifyRows, hipHostMallocDefault));
  *out = ctx.release();
  return ok();
}

namespace speca {
LaneSplit split_lanes(const speca_ctx* ctx, int n, int min_rows) {
  LaneSplit ls;
  int k = ctx->lanes;
  if (ctx->prof.on && !ctx->prof.keep_lanes) k = 1;
  if (min_rows < 1) min_rows = 1;
  while (k > 1 && n / k < min_rows) --k;
  ls.n_lanes = k;
  for (int i = 0; i <= k; ++i) ls.first[i] = static_cast<int>(static_cast<int64_t>(n) * i / k);
  return ls;
}
Error lanes_fork(speca_ctx* ctx, const LaneSplit& ls) {
  if (ls.n_lanes <= 1) return ok();
  SPECA_HIP(hipEventRecord(ctx->lane_fork, ctx->stream));
  for (int k = 1; k < ls.n_lanes; ++k) SPECA_HIP(hipStreamWaitEvent(ctx->lane_stream[k], ctx->lane_fork, 0));
  return ok();
}
Error lanes_join(speca_ctx* ctx, const LaneSplit& ls) {
  for (int k = 1; k < ls.n_lanes; ++k) {
    SPECA_HIP(hipEventRecord(ctx->lane_join[k], ctx->lane_stream[k]));
    SPECA_HIP(hipStreamWaitEvent(ctx->stream, ctx->lane_join[k], 0));
  }
  return ok();
}
RowTable slice_table(const RowTable& rt, int first, int n) {
  RowTable o{};
  o.n = n;
  for (int i = 0; i < n; ++i) {
    o.row[i] = rt.row[first + i];
    o.order[i] = rt.order[first + i];
    for (int q = 0; q < kMaxTensors; ++q) o.w[i][q] = rt.w[first + i][q];
  }
  return o;
}
}  // namespace speca

static Error init_cache_impl(speca_ctx* ctx, const speca_cfg* cfg, int batch_rows) {
  std::string why;
  if (!cfg_ok(cfg, &why)) SPECA_FAIL(SPECA_EINVAL, "%s", why.c_str());
  if (batch_rows < 1) SPECA_FAIL(SPECA_EINVAL, "batch_rows = %d", batch_rows);
  const int n_slots = ctx->model ? ctx->model->n_slots() : ctx->desc.n_slots;
  const int n_blocks = ctx->model ? ctx->model->n_blocks() : n_slots;
  const int64_t tokens = ctx->model ? ctx->model->tokens() : ctx->desc.tokens;
  if (cfg->verify_block >= n_blocks) SPECA_FAIL(SPECA_EINVAL, "verify_block = %d but the model has %d blocks", cfg->verify_block, n_blocks);
  CacheGeom g{};
  g.E = tokens * ctx->desc.hidden;
  g.n_slots = n_slots;
  g.m = cfg->order;
  g.batch_rows = batch_rows;
  g.dtype = ctx->desc.dtype;
  const size_t bytes = static_cast<size_t>(g.E) * n_slots * (cfg->order + 1) * batch_rows * dtype_size(g.dtype);
  if (bytes > ctx->cache_cap) {
    if (ctx->geom.base) {
      SPECA_HIP(hipStreamSynchronize(ctx->stream));
      SPECA_HIP(hipFree(ctx->geom.base));
      ctx->geom.base = nullptr;
      ctx->cache_cap = 0;
      ctx->cache_ready = false;
    }
    void* p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) {
      (void)hipGetLastError();
      SPECA_FAIL(SPECA_ENOMEM, "cannot allocate %zu bytes of feature cache", bytes);
    }
    ctx->geom.base = p;
    ctx->cache_cap = bytes;
  }
  g.base = ctx->geom.base;
  ctx->geom = g;
  ctx->cfg = *cfg;
  ctx->batch_rows = batch_rows;
  clear_refs(ctx);
  if (ctx->model) {
    SPECA_TRY(ctx->model->prepare(ctx, batch_rows));
    const size_t mo = static_cast<size_t>(batch_rows) * ctx->model->latent_elems() * sizeof(float);
    if (mo > ctx->model_out_cap) {
      if (ctx->model_out) {
        SPECA_HIP(hipStreamSynchronize(ctx->stream));
        SPECA_HIP(hipFree(ctx->model_out));
        ctx->model_out = nullptr;
        ctx->model_out_cap = 0;
      }
      if (hipMalloc(reinterpret_cast<void**>(&ctx->model_out), mo) != hipSuccess) {
        (void)hipGetLastError();
        SPECA_FAIL(SPECA_ENOMEM, "cannot allocate %zu bytes for the model outputs of a step", mo);
      }
      ctx->model_out_cap = mo;
    }
  }
  ctx->cache_ready = true;
  return ok();
}

static Error refresh_impl(speca_ctx* ctx, int step, const int32_t* rows, int n_rows, const void* features) {
  if (!ctx->cache_ready) SPECA_FAIL(SPECA_ESTATE, "speca_init_cache has not been called");
  if (!features) SPECA_FAIL(SPECA_EINVAL, "features is NULL");
  if (step < 0) SPECA_FAIL(SPECA_EINVAL, "step = %d", step);
  SPECA_TRY(check_rows(ctx, rows, n_rows));
  if (n_rows > kMaxRows) SPECA_FAIL(SPECA_EUNSUPPORTED, "speca_refresh takes at most %d rows per call", kMaxRows);
  RowTable rt;
  SPECA_TRY(build_refresh_table(ctx, step, rows, n_rows, &rt));
  {
    // reads the new feature and the old differences below the new order, writes the new differences
    const double esz = dtype_size(ctx->geom.dtype);
    ProfScope ps(ctx, SPECA_PROF_REFRESH, 0.0, ctx->geom.n_slots * ctx->geom.E * esz * (2.0 * table_tensors(rt)));
    SPECA_TRY(launch_refresh(ctx->geom, rt, features, ctx->stream));
  }
  push_refs(ctx, step, rows, n_rows);
  return ok();
}

static Error forecast_impl(speca_ctx* ctx, int step, const int32_t* rows, int n_rows, void* out) {
  if (!ctx->cache_ready) SPECA_FAIL(SPECA_ESTATE, "speca_init_cache has not been called");
  if (!out) SPECA_FAIL(SPECA_EINVAL, "out_features is NULL");
  SPECA_TRY(check_rows(ctx, rows, n_rows));
  if (n_rows > kMaxRows) SPECA_FAIL(SPECA_EUNSUPPORTED, "speca_forecast takes at most %d rows per call", kMaxRows);
  RowTable rt;
  SPECA_TRY(build_forecast_table(ctx, step, rows, n_rows, &rt));
  const double esz = dtype_size(ctx->geom.dtype);
  ProfScope ps(ctx, SPECA_PROF_FORECAST, 0.0, ctx->geom.n_slots * ctx->geom.E * esz * (table_tensors(rt) + rt.n));
  return launch_forecast(ctx->geom, rt, out, ctx->stream);
}

static Error verify_impl(speca_ctx* ctx, const void* pred, const void* truth, int n_rows, int64_t E, int dtype,
                         const float* tau, float eps, float* err_out, uint8_t* accept_out) {
  if (!pred || !truth || !err_out) SPECA_FAIL(SPECA_EINVAL, "pred, truth and err_out must not be NULL");
  if (tau && !accept_out) SPECA_FAIL(SPECA_EINVAL, "accept_out is NULL but tau_per_row is given");
  if (n_rows < 1) SPECA_FAIL(SPECA_EINVAL, "n_rows = %d", n_rows);
  if (E < 1) SPECA_FAIL(SPECA_EINVAL, "elems_per_row = %lld", static_cast<long long>(E));
  if (dtype != SPECA_F32 && dtype != SPECA_BF16) SPECA_FAIL(SPECA_EINVAL, "dtype = %d", dtype);
  if (!(eps >= 0.0f)) SPECA_FAIL(SPECA_EINVAL, "eps < 0");
  const int metric = ctx->cache_ready ? ctx->cfg.metric : SPECA_METRIC_L2;
  const size_t esz = dtype_size(dtype);
  VerifyScratch& v = ctx->vs;
  for (int r0 = 0; r0 < n_rows; r0 += kMaxVerifyRows) {
    const int n = std::min(kMaxVerifyRows, n_rows - r0);
    SPECA_TRY(ensure_partial(ctx, static_cast<size_t>(n) * verify_chunks(E) * 3));
    if (tau) {
      std::memcpy(v.h_tau, tau + r0, n * sizeof(float));
      SPECA_HIP(hipMemcpyAsync(v.tau_dev, v.h_tau, n * sizeof(float), hipMemcpyHostToDevice, ctx->stream));
    }
    const char* p = static_cast<const char*>(pred) + static_cast<size_t>(r0) * E * esz;
    const char* t = static_cast<const char*>(truth) + static_cast<size_t>(r0) * E * esz;
    {
      ProfScope ps(ctx, SPECA_PROF_VERIFY, 0.0, 2.0 * n * E * esz);
      SPECA_TRY(launch_verify(metric, p, dtype, t, dtype, E, nullptr, nullptr, 0, n, eps, tau ? v.tau_dev : nullptr, v.partial,
                              v.err_dev, v.acc_dev, ctx->stream));
    }
    SPECA_HIP(hipMemcpyAsync(v.h_err, v.err_dev, n * sizeof(float), hipMemcpyDeviceToHost, ctx->stream));
    if (tau) SPECA_HIP(hipMemcpyAsync(v.h_acc, v.acc_dev, n, hipMemcpyDeviceToHost, ctx->stream));
    SPECA_HIP(hipStreamSynchronize(ctx->stream));
    std::memcpy(err_out + r0, v.h_err, n * sizeof(float));
    if (tau) std::memcpy(accept_out + r0, v.h_acc, n);
  }
  return ok();
}

// Eq. 4 with device-side inputs and outputs and the file-scope scratch: no allocation, no synchronisation.
static Error verify_static_impl(speca_ctx* ctx, const void* pred, const void* truth, int n_rows, int64_t E, int dtype,
                                const float* tau_dev, float eps, float* err_dev, uint8_t* accept_dev) {
  if (!pred || !truth || !err_dev) SPECA_FAIL(SPECA_EINVAL, "pred, truth and err_out must not be NULL");
  if (tau_dev && !accept_dev) SPECA_FAIL(SPECA_EINVAL, "accept_out is NULL but tau_per_row is given");
  if (n_rows < 1) SPECA_FAIL(SPECA_EINVAL, "n_rows = %d", n_rows);
  if (E < 1) SPECA_FAIL(SPECA_EINVAL, "elems_per_row = %lld", static_cast<long long>(E));
  if (dtype != SPECA_F32 && dtype != SPECA_BF16) SPECA_FAIL(SPECA_EINVAL, "dtype = %d", dtype);
  if (!(eps >= 0.0f)) SPECA_FAIL(SPECA_EINVAL, "eps < 0");
  const int64_t chunks = verify_chunks(E);
  const int64_t per_launch = std::min<int64_t>(n_rows, kMaxRows) * chunks;
  if (per_launch > SPECA_VERIFY_STATIC_MAX_PARTIALS)
    SPECA_FAIL(SPECA_EINVAL, "speca_verify_static: %lld partial sums per launch (%d rows x %lld chunks) exceed the static scratch of %d",
               static_cast<long long>(per_launch), std::min(n_rows, kMaxRows), static_cast<long long>(chunks), SPECA_VERIFY_STATIC_MAX_PARTIALS);
  if (!ctx->static_partial) SPECA_FAIL(SPECA_ESTATE, "the static scratch was not resolved at create");
  const int metric = ctx->cache_ready ? ctx->cfg.metric : SPECA_METRIC_L2;
  const size_t esz = dtype_size(dtype);
  // row groups of one call reuse the scratch one after the other: same stream, so in order
  for (int r0 = 0; r0 < n_rows; r0 += kMaxRows) {
    const int n = std::min(kMaxRows, n_rows - r0);
    const char* p = static_cast<const char*>(pred) + static_cast<size_t>(r0) * E * esz;
    const char* t = static_cast<const char*>(truth) + static_cast<size_t>(r0) * E * esz;
    SPECA_TRY(launch_verify(metric, p, dtype, t, dtype, E, nullptr, nullptr, 0, n, eps, tau_dev ? tau_dev + r0 : nullptr, ctx->static_partial,
                            err_dev + r0, accept_dev ? accept_dev + r0 : nullptr, ctx->stream));
  }
  return ok();
}

static Error labels_for_rows(const speca_ctx* ctx, const speca_cond* cond, std::vector<int32_t>* out) {
  out->assign(ctx->batch_rows, 0);
  if (ctx->desc.kind == SPECA_MODEL_DIT) {
    if (!cond->labels) SPECA_FAIL(SPECA_EINVAL, "cond->labels is NULL");
    for (int r = 0; r < ctx->batch_rows; ++r) {
      if (cond->labels[r] < 0 || cond->labels[r] > ctx->desc.num_classes)
        SPECA_FAIL(SPECA_EINVAL, "label %d of row %d out of range", cond->labels[r], r);
      (*out)[r] = cond->labels[r];
    }
  }
  return ok();
}

static Error full_step_impl(speca_ctx* ctx, const void* x, const speca_cond* cond, int step, const int32_t* rows, int n_rows,
                            void* model_out) {
  if (!ctx->model) SPECA_FAIL(SPECA_EUNSUPPORTED, "this context has no model (cache-only)");
  if (!ctx->cache_ready) SPECA_FAIL(SPECA_ESTATE, "speca_init_cache has not been called");
  if (!x || !cond || !model_out) SPECA_FAIL(SPECA_EINVAL, "x, cond and model_out must not be NULL");
  if (step < 0) SPECA_FAIL(SPECA_EINVAL, "step = %d", step);
  SPECA_TRY(check_rows(ctx, rows, n_rows));
  for (int i = 0; i < n_rows; ++i) {
    const RefHistory& h = ctx->row_refs[rows[i]];
    if (h.n > 0 && step <= h.r[0]) SPECA_FAIL(SPECA_ESTATE, "step %d is not after row %d's latest reference %d", step, rows[i], h.r[0]);
  }
  std::vector<int32_t> labels;
  SPECA_TRY(labels_for_rows(ctx, cond, &labels));
  SPECA_TRY(ctx->model->full_step(ctx, static_cast<const float*>(x), ctx->batch_rows, cond, labels.data(), step, rows, n_rows,
                                  static_cast<float*>(model_out)));
  return ok();
}

static Error spec_step_impl(speca_ctx* ctx, const void* x, const speca_cond* cond, int step, const int32_t* rows, int n_rows,
                            const float* tau, int pair_stride, float* err_out, uint8_t* accept_out, void* model_out) {
  if (!ctx->model) SPECA_FAIL(SPECA_EUNSUPPORTED, "this context has no model (cache-only)");
  if (!ctx->cache_ready) SPECA_FAIL(SPECA_ESTATE, "speca_init_cache has not been called");
  if (!x || !cond || !model_out || !tau || !err_out || !accept_out) SPECA_FAIL(SPECA_EINVAL, "NULL argument");
  SPECA_TRY(check_rows(ctx, rows, n_rows));
  if (n_rows > kMaxRows) SPECA_FAIL(SPECA_EUNSUPPORTED, "speca_spec_step takes at most %d rows per call", kMaxRows);
  if (pair_stride < 0) SPECA_FAIL(SPECA_EINVAL, "pair_stride = %d", pair_stride);
  std::vector<int32_t> labels;
  SPECA_TRY(labels_for_rows(ctx, cond, &labels));
  SPECA_TRY(ctx->model->spec_step(ctx, static_cast<const float*>(x), ctx->batch_rows, cond, labels.data(), step, rows, n_rows,
                                  tau, pair_stride, static_cast<float*>(model_out)));
  std::memcpy(err_out, ctx->vs.h_err, n_rows * sizeof(float));
  std::memcpy(accept_out, ctx->vs.h_acc, n_rows);
  return ok();
}

namespace speca {
Error sample_impl(speca_ctx* ctx, float* latents, int batch, const speca_cond* cond, const speca_solver* solver, const float* tau,
                  speca_trace* trace);
}

extern "C" {

int speca_create(speca_ctx** out, const speca_model_desc* desc, const speca_weights* w, void* hip_stream) {
  if (!out) { g_create_error = "out is NULL"; return SPECA_EINVAL; }
  *out = nullptr;
  speca_ctx* ctx = nullptr;
  Error e = create_impl(&ctx, desc, w, hip_stream);
  if (e.code != SPECA_OK) { g_create_error = e.msg; return e.code; }
  *out = ctx;
  return SPECA_OK;
}

int speca_destroy(speca_ctx* ctx) {
  free_ctx(ctx);
  return SPECA_OK;
}

const char* speca_last_error(const speca_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

int speca_set_lanes(speca_ctx* ctx, int lanes, int profile_keeps_lanes) {
  if (!ctx) return SPECA_EINVAL;
  if (lanes < 1 || lanes > kMaxLanes) return finish(ctx, [&]() -> Error { SPECA_FAIL(SPECA_EINVAL, "lanes = %d (1..%d)", lanes, kMaxLanes); }());
  ctx->lanes = lanes;
  ctx->prof.keep_lanes = profile_keeps_lanes != 0;
  return SPECA_OK;
}

int speca_init_cache(speca_ctx* ctx, const speca_cfg* cfg, int batch_rows) {
  if (!ctx) return SPECA_EINVAL;
  return finish(ctx, init_cache_impl(ctx, cfg, batch_rows));
}

int speca_refresh(speca_ctx* ctx, int step, const int32_t* rows, int n_rows, const void* features) {
  if (!ctx) return SPECA_EINVAL;
  return finish(ctx, refresh_impl(ctx, step, rows, n_rows, features));
}

int speca_full_step(speca_ctx* ctx, const void* x, const speca_cond* cond, int step, const int32_t* rows, int n_rows,
                    void* model_out) {
  if (!ctx) return SPECA_EINVAL;
  return finish(ctx, full_step_impl(ctx, x, cond, step, rows, n_rows, model_out));
}

int speca_forecast(speca_ctx* ctx, int step, const int32_t* rows, int n_rows, void* out_features) {
  if (!ctx) return SPECA_EINVAL;
  return finish(ctx, forecast_impl(ctx, step, rows, n_rows, out_features));
}

int speca_verify(speca_ctx* ctx, const void* pred, const void* truth, int n_rows, int64_t elems_per_row, int dtype,
                 const float* tau_per_row, float eps, float* err_out, uint8_t* accept_out) {
  if (!ctx) return SPECA_EINVAL;
  return finish(ctx, verify_impl(ctx, pred, truth, n_rows, elems_per_row, dtype, tau_per_row, eps, err_out, accept_out));
}

int speca_verify_static(speca_ctx* ctx, const void* pred, const void* truth, int n_rows, int64_t elems_per_row, int dtype,
                        const float* tau_per_row, float eps, float* err_out, uint8_t* accept_out) {
  if (!ctx) return SPECA_EINVAL;
  return finish(ctx, verify_static_impl(ctx, pred, truth, n_rows, elems_per_row, dtype, tau_per_row, eps, err_out, accept_out));
}

int speca_spec_step(speca_ctx* ctx, const void* x, const speca_cond* cond, int step, const int32_t* rows, int n_rows,
                    const float* tau_per_row, int pair_stride, float* err_out, uint8_t* accept_out, void* model_out) {
  if (!ctx) return SPECA_EINVAL;
  return finish(ctx, spec_step_impl(ctx, x, cond, step, rows, n_rows, tau_per_row, pair_stride, err_out, accept_out, model_out));
}

int speca_linear(void* hip_stream, int dtype, const void* a, int m, int k, const void* w, int n, const void* bias, int act,
                 void* out) {
  if (dtype != SPECA_F32 && dtype != SPECA_BF16) { g_create_error = "dtype"; return SPECA_EINVAL; }
  if (!a || !w || !out || m < 1 || n < 1 || k < 1 || act < 0 || act > 2) { g_create_error = "speca_linear: bad argument"; return SPECA_EINVAL; }
  GemmEpi e;
  e.mode = act == 1 ? EPI_GELU : act == 2 ? EPI_SILU : EPI_STORE;
  e.bias = bias; e.out = out; e.ldo = n;
  Error r = launch_gemm(dtype, a, k, w, k, m, n, k, e, static_cast<hipStream_t>(hip_stream));
  if (r.code != SPECA_OK) g_create_error = r.msg;
  return r.code;
}

int speca_attention(void* hip_stream, int dtype, const void* qkv, void* out, int rows, int tokens, int heads, int head_dim) {
  if (dtype != SPECA_F32 && dtype != SPECA_BF16) { g_create_error = "dtype"; return SPECA_EINVAL; }
  Error r = launch_attention(dtype, qkv, out, static_cast<int64_t>(heads) * head_dim, rows, tokens, heads, head_dim, static_cast<hipStream_t>(hip_stream));
  if (r.code != SPECA_OK) g_create_error = r.msg;
  return r.code;
}

int speca_profile_begin(speca_ctx* ctx) {
  if (!ctx) return SPECA_EINVAL;
  for (auto& r : ctx->prof.recs) { ctx->prof.pool.push_back(r.a); ctx->prof.pool.push_back(r.b); }
  ctx->prof.recs.clear();
  ctx->prof.on = true;
  return SPECA_OK;
}

int speca_profile_end(speca_ctx* ctx, speca_profile* out) {
  if (!ctx || !out) return SPECA_EINVAL;
  ctx->prof.on = false;
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) { ctx->err = "hipStreamSynchronize failed"; return SPECA_EHIP; }
  std::memset(out, 0, sizeof(*out));
  for (auto& r : ctx->prof.recs) {
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) { ctx->err = "hipEventElapsedTime failed"; return SPECA_EHIP; }
    out->launches[r.cls] += 1;
    out->ms[r.cls] += ms;
    out->flops[r.cls] += r.flops;
    out->bytes[r.cls] += r.bytes;
    ctx->prof.pool.push_back(r.a);
    ctx->prof.pool.push_back(r.b);
  }
  ctx->prof.recs.clear();
  return SPECA_OK;
}

int speca_sample(speca_ctx* ctx, void* latents_inout, int batch, const speca_cond* cond, const speca_solver* solver,
                 const float* tau, speca_trace* trace_out) {
  if (!ctx) return SPECA_EINVAL;
  return finish(ctx, sample_impl(ctx, static_cast<float*>(latents_inout), batch, cond, solver, tau, trace_out));
}

}  // extern "C"
