/*
 * speca.h - C ABI of the MI355X (gfx950) SpeCa sampling-step library.
 *
 * SpeCa ("forecast-then-verify" sampling for diffusion transformers):
 *   (1) at a reference step the model runs in full and a per-slot cache of branch
 *       features and their finite differences is refreshed (Sec. 3.2 step 1; Sec. 3.3, Eq. 3);
 *   (2) at speculative steps every cached feature is forecast by a Taylor-series
 *       combination of those differences (Sec. 3.3, Eq. 2);
 *   (3) the forecast is verified at one deep block: that block is recomputed for real,
 *       the relative L2 error between forecast and recomputed feature is compared with
 *       a step-dependent threshold, the sample is accepted or falls back to full
 *       compute (Sec. 3.4, Eq. 4, sequential validation, adaptive threshold).
 *
 * Conventions
 *   - "step" s = 0..S-1 counts sampling steps upwards (the paper's timestep t decreases).
 *   - A "row" is one sequence of the model's batch.  With classifier-free guidance a
 *     sample owns two rows (conditional b, unconditional B+b).
 *   - A "slot" is one cached branch output [rows, tokens, hidden]: DiT blocks own two
 *     (attention branch, MLP branch) in block order.
 *   - DEVICE pointers are raw HIP device addresses owned by the caller (e.g. torch
 *     tensors) unless stated otherwise; HOST pointers are ordinary process memory.
 *   - Every function returns a speca_status; it never throws or aborts.  The message of
 *     the last failure on a context is available from speca_last_error().
 *   - All device work of a context is enqueued on the HIP stream given at creation, or on
 *     library-owned streams forked from and joined back to it inside a call (speca_set_lanes),
 *     so a caller sees ordinary stream order on that stream.
 *     Calls that return host results (speca_verify, speca_spec_step, speca_sample)
 *     synchronise that stream before returning; the others are asynchronous.
 *   - A context is not thread-safe; contexts are independent of each other.
 */
#ifndef SPECA_H
#define SPECA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct speca_ctx speca_ctx;

typedef enum speca_status {
  SPECA_OK = 0,
  SPECA_EINVAL = 1,        /* bad argument (null pointer, size, enum, row index) */
  SPECA_ENOMEM = 2,        /* device or host allocation failed */
  SPECA_ESTATE = 3,        /* call order: cache not initialised, row without a reference, ... */
  SPECA_EHIP = 4,          /* a HIP runtime call or kernel launch failed */
  SPECA_EUNSUPPORTED = 5   /* valid request this build does not implement */
} speca_status;

enum { SPECA_F32 = 0, SPECA_BF16 = 1 };                       /* storage types */
enum { SPECA_MODEL_NONE = 0, SPECA_MODEL_DIT = 1, SPECA_MODEL_MMDIT = 2 };
enum { SPECA_COEF_TAYLOR = 0, SPECA_COEF_NEWTON = 1, SPECA_COEF_ADAMS_BASHFORTH = 2 };
enum { SPECA_SOLVER_DDIM = 0, SPECA_SOLVER_FLOW = 1, SPECA_SOLVER_DDPM = 2 };
enum { SPECA_KIND_FULL = 0, SPECA_KIND_SPEC = 1, SPECA_KIND_REJECT = 2 };
enum { SPECA_METRIC_L2 = 0, SPECA_METRIC_L1 = 1, SPECA_METRIC_LINF = 2, SPECA_METRIC_COSINE = 3 };
/* What the m+1 planes of a cache slot hold.  DIFFERENCES: D^0 .. D^m of Eq. 3, updated by the recursion at
 * every full step (the layout Sec. 3.3 describes).  RING: the features of the last m+1 full steps, each stored
 * once and never re-read by a refresh; the differences are linear in them, so a forecast (Eq. 2) is a weighted
 * sum of the planes with weights the host derives from the same recursion (speca_ring_weights).  Both give
 * the same forecasts in exact arithmetic; they differ in what is rounded to the cache type (differences /
 * features) and in refresh traffic (reads m, writes m+1 planes / writes one). */
enum { SPECA_CACHE_DIFFERENCES = 0, SPECA_CACHE_RING = 1 };

#define SPECA_MAX_ORDER 4          /* highest Taylor order m the cache can hold */
#define SPECA_MAX_LAUNCH_ROWS 64   /* rows handled by one internal launch; larger lists are chunked */

/* Shape of the target model (Sec. 3.1.2 names the architecture; sizes are the caller's).
 * kind NONE describes a bare cache (n_slots x tokens x hidden) with no model attached:
 * only init_cache / refresh / forecast / verify are available on such a context. */
typedef struct speca_model_desc {
  int32_t kind;            /* SPECA_MODEL_* */
  int32_t dtype;           /* SPECA_F32 | SPECA_BF16: weights, activations, cache */
  int32_t depth;           /* DiT: blocks.  MMDiT: dual-stream blocks */
  int32_t depth_single;    /* MMDiT: single-stream blocks (0 for DiT) */
  int32_t hidden;          /* D */
  int32_t heads;           /* H; head_dim = D / H */
  int32_t mlp_hidden;      /* Dm */
  int32_t in_channels;     /* latent channels C */
  int32_t latent_t;        /* latent frames (1 for images) */
  int32_t latent_h;
  int32_t latent_w;
  int32_t patch;           /* spatial patch p (tokens = t * h/p * w/p) */
  int32_t num_classes;     /* DiT: label table has num_classes+1 rows, the last is the null label */
  int32_t freq_dim;        /* width of the sinusoidal timestep embedding */
  int32_t txt_tokens;      /* MMDiT */
  int32_t txt_dim;         /* MMDiT */
  int32_t vec_dim;         /* MMDiT pooled-conditioning width */
  int32_t n_slots;         /* kind NONE only */
  int32_t tokens;          /* kind NONE only */
} speca_model_desc;

/* Table of caller-owned DEVICE tensors, looked up by name ("blk3.qkv_w", ...).
 * Linear weights are [out_features, in_features] row-major in the model dtype.
 * numel[i] is checked against the shape the descriptor implies. */
typedef struct speca_weights {
  int32_t count;
  const char* const* names;     /* HOST */
  const void* const* ptrs;      /* HOST array of DEVICE pointers */
  const int64_t* numel;         /* HOST */
} speca_weights;

/* SpeCa hyper-parameters (Sec. 3.3: order m, interval N; Sec. 3.4: eps; appendix:
 * forced activation period, verify layer). */
typedef struct speca_cfg {
  int32_t order;           /* m, 0..SPECA_MAX_ORDER */
  int32_t interval;        /* N >= 1: a full step is forced once step - last_full >= N */
  int32_t verify_block;    /* block recomputed for verification; -1 = last block */
  int32_t coef_mode;       /* SPECA_COEF_TAYLOR (Eq. 2 as printed) | SPECA_COEF_NEWTON | SPECA_COEF_ADAMS_BASHFORTH */
  float   eps;             /* Eq. 4 epsilon, paper value 1e-8 */
  int32_t warmup_full;     /* steps 0..warmup_full-1 are always full (>= 1) */
  int32_t metric;          /* SPECA_METRIC_*; L2 is Eq. 4 */
  int32_t layout;          /* SPECA_CACHE_DIFFERENCES (Sec. 3.3 as described) | SPECA_CACHE_RING */
} speca_cfg;

/* Conditioning of one call. */
typedef struct speca_cond {
  const int32_t* labels;   /* HOST.  DiT: one class label per row (per sample for speca_sample) */
  const void* txt;         /* DEVICE. MMDiT text tokens [rows, txt_tokens, txt_dim], model dtype */
  const void* pooled;      /* DEVICE. MMDiT pooled vector [rows, vec_dim], model dtype */
  float timestep;          /* value the model is conditioned on (ignored by speca_sample) */
} speca_cond;

/* Solver tables are data (the method is independent of the noise schedule). */
typedef struct speca_solver {
  int32_t kind;            /* SPECA_SOLVER_DDIM (eta = 0) | SPECA_SOLVER_FLOW (Euler) | SPECA_SOLVER_DDPM (Eq. 1) */
  int32_t steps;           /* S */
  const float* timesteps;  /* HOST [S]   conditioning value of step s */
  const float* table;      /* HOST [S+1] alpha_bar (DDIM, DDPM; last entry 1) or sigma (flow; last entry 0) */
  float cfg_scale;         /* > 0: classifier-free guidance, rows = 2 x batch, null label for the second half */
  const float* noise;      /* DEVICE fp32 [S][batch, C, (T,) H, W]: the standard-normal draws of DDPM (the library
                            * draws nothing itself, so a trajectory is a function of its inputs); step S-1 is not
                            * read.  Ignored by the other solvers; NULL with DDPM is SPECA_EINVAL.
                            * DDPM step, Eq. 1 on the given (possibly sub-sampled) schedule:
                            *   alpha = table[s] / table[s+1], beta = 1 - alpha,
                            *   x <- (x - beta / sqrt(1 - table[s]) * e) / sqrt(alpha) + sqrt(beta) * noise[s];
                            * the final step returns the mean. */
} speca_solver;

/* Per-sample, per-step record of speca_sample.  All HOST memory owned by the caller;
 * any pointer may be NULL. */
typedef struct speca_trace {
  int8_t* kind;            /* [batch][S]      SPECA_KIND_* */
  float*  err;             /* [batch][S][2]   Eq. 4 error per row of the sample (NaN = not verified / no second row) */
  int32_t n_full;          /* out: sample-steps computed in full (scheduled or after a rejection) */
  int32_t n_spec;          /* out: sample-steps accepted */
  int32_t n_reject;        /* out: speculative attempts rejected */
} speca_trace;

/* ---- life cycle ------------------------------------------------------------------- */

/* Create a context for `desc` with weights `w` (may be NULL for kind NONE) on HIP stream
 * `hip_stream` (a hipStream_t; NULL = the null stream).  The weight tensors must outlive
 * the context.  Allocates no cache yet. */
int speca_create(speca_ctx** out, const speca_model_desc* desc, const speca_weights* w, void* hip_stream);
int speca_destroy(speca_ctx* ctx);
/* Message of the last failed call on ctx (ctx == NULL: of the last failed create). */
const char* speca_last_error(const speca_ctx* ctx);

/* ---- (1) cache --------------------------------------------------------------------- */

/* Allocate (or re-use) and reset the cache [slot][order 0..m][batch_rows][tokens][hidden]
 * and the per-row reference history; also sizes the activation workspace for batch_rows.
 * May be called again to start a new trajectory.  Sec. 3.3 (features + differences). */
int speca_init_cache(speca_ctx* ctx, const speca_cfg* cfg, int batch_rows);

/* (With cfg.layout = SPECA_CACHE_RING the planes hold raw features: speca_refresh stores F into the row's
 * next plane and nothing else; speca_forecast and every fused path weight the planes accordingly.)
 * Cache refresh from materialised features (the cache-only form of a reference step):
 * features is DEVICE [n_slots][n_rows][tokens][hidden] in the cache dtype, row i of it
 * belongs to cache row rows[i] (HOST, strictly increasing).  For every listed row stores
 * D0 <- F and D^i <- (D^{i-1}_new - D^{i-1}_old) / d_i, i <= min(m, #references so far),
 * then records `step` as the row's latest reference.  d_i = step - last reference
 * (TAYLOR; with a uniform gap N this is Eq. 3 scaled by N^-i) or step - i-th last
 * reference (NEWTON).  step must exceed the row's latest reference.  Asynchronous. */
int speca_refresh(speca_ctx* ctx, int step, const int32_t* rows, int n_rows, const void* features);

/* ---- (2) reference step ---------------------------------------------------------------- */

/* Full forward of the model for the listed rows at sampling step `step`, with cache
 * refresh fused into the branch epilogues.  x: DEVICE fp32 [batch_rows, C, (T,) H, W]
 * (all rows present; only the listed ones are read).  model_out: DEVICE fp32, same shape;
 * only the listed rows are written.  Sec. 3.2 step 1.  Asynchronous. */
int speca_full_step(speca_ctx* ctx, const void* x, const speca_cond* cond, int step,
                    const int32_t* rows, int n_rows, void* model_out);

/* ---- (3) forecast ---------------------------------------------------------------------- */

/* Eq. 2 for every slot of the listed rows at distance k = step - latest reference of the
 * row (each row may have its own k and its own available order).  out_features: DEVICE
 * [n_slots][n_rows][tokens][hidden] in the cache dtype.  A row without a reference, or
 * with step <= its latest reference, is SPECA_ESTATE.  Asynchronous. */
int speca_forecast(speca_ctx* ctx, int step, const int32_t* rows, int n_rows, void* out_features);

/* ---- (4) verification ------------------------------------------------------------------ */

/* Eq. 4 on two DEVICE tensors [n_rows][elems_per_row] of type dtype:
 * err[r] = ||pred_r - truth_r||_2 / (||truth_r||_2 + eps) (or the cfg metric), fp32, fixed
 * summation order (bit-reproducible, independent of n_rows); accept[r] = err[r] <= tau[r].
 * tau_per_row, err_out, accept_out are HOST arrays of n_rows; tau_per_row may be NULL
 * (then accept_out is not written).  Synchronises. */
int speca_verify(speca_ctx* ctx, const void* pred, const void* truth, int n_rows, int64_t elems_per_row,
                 int dtype, const float* tau_per_row, float eps, float* err_out, uint8_t* accept_out);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The same reduction as speca_verify (same kernels, same fixed summation order, so the same bits)
 * with everything on the device and nothing allocated or synchronised: tau_per_row (may be NULL: then
 * accept_out is not written), err_out and accept_out are DEVICE arrays of n_rows owned by the caller; the call
 * is asynchronous on the context's stream and makes no HIP allocation, free or copy.  The stage-1 partial sums
 * live in a file-scope device array of SPECA_VERIFY_STATIC_MAX_PARTIALS x 3 floats (768 KiB, held by every GPU
 * the library runs on until the process ends): min(n_rows, SPECA_MAX_LAUNCH_ROWS) x ceil(elems_per_row / 8192)
 * must not exceed SPECA_VERIFY_STATIC_MAX_PARTIALS, else SPECA_EINVAL with a message and nothing is launched.
 * Every partial is written before it is read, so nothing in the array needs clearing between calls.  All
 * contexts on one GPU share the array: calls that overlap in time on one GPU (different streams or threads)
 * race; calls on one stream are ordered and safe. */
#define SPECA_VERIFY_STATIC_MAX_PARTIALS 65536
int speca_verify_static(speca_ctx* ctx, const void* pred, const void* truth, int n_rows, int64_t elems_per_row,
                        int dtype, const float* tau_per_row, float eps, float* err_out, uint8_t* accept_out);

/* Speculative attempt (Sec. 3.2 steps 2-3) for the listed rows at `step`: forecast all
 * slots and fold them, gated by the step's own modulation, into the hidden state up to
 * the verify block; run the verify block for real; Eq. 4 between the forecast and the
 * recomputed last slot of that block; rows whose error passes tau_per_row are finished
 * with forecasts for all remaining blocks and their model_out rows are written.  With
 * pair_stride > 0 rows r and r + pair_stride (both must be listed) are accepted only
 * together.  err_out / accept_out: HOST [n_rows].  The cache is not modified.  Synchronises. */
int speca_spec_step(speca_ctx* ctx, const void* x, const speca_cond* cond, int step,
                    const int32_t* rows, int n_rows, const float* tau_per_row, int pair_stride,
                    float* err_out, uint8_t* accept_out, void* model_out);

/* ---- (5) whole trajectory -------------------------------------------------------------- */

/* SpeCa sampling of `batch` samples (batch_rows of the cache must be batch, or 2*batch
 * with guidance): per step each sample is scheduled full or speculative, speculative
 * samples are verified against tau[step], rejected ones are recomputed in full at the
 * same step, then the solver update is applied.  tau[s] <= 0 makes step s full.
 * latents_inout: DEVICE fp32 [batch, C, (T,) H, W], overwritten with the final latents.
 * tau: HOST [S].  Re-initialises the cache state.  Synchronises. */
int speca_sample(speca_ctx* ctx, void* latents_inout, int batch, const speca_cond* cond,
                 const speca_solver* solver, const float* tau, speca_trace* trace_out);


/* ---- the dense contractions of the reference step, callable on their own ------------------- */

/* out[m][n] = act(sum_k a[m][k] w[n][k] + bias[n]) on DEVICE tensors of type dtype (a: [m][k],
 * w: [n][k], bias: [n] or NULL, out: [m][n]); act 0 = none, 1 = GELU (tanh form), 2 = SiLU;
 * fp32 accumulation.  These are the QKV / out-proj / MLP GEMMs of a block (Sec. 3.1.2) at
 * whatever shape the caller gives; n must be a multiple of 4.  Asynchronous on hip_stream.
 * Errors: message via speca_last_error(NULL). */
int speca_linear(void* hip_stream, int dtype, const void* a, int m, int k, const void* w, int n, const void* bias, int act,
                 void* out);
/* out = softmax(q k^T / sqrt(head_dim)) v without mask; qkv: DEVICE [rows][tokens][3][heads][head_dim],
 * out: DEVICE [rows][tokens][heads*head_dim], both of type dtype.  Asynchronous on hip_stream. */
int speca_attention(void* hip_stream, int dtype, const void* qkv, void* out, int rows, int tokens, int heads, int head_dim);

/* ---- measurement ----------------------------------------------------------------------------- */

/* Kernel classes of the per-class timing below. */
enum { SPECA_PROF_GEMM = 0,      /* QKV / out-proj / FC1 / FC2 contractions of the blocks */
       SPECA_PROF_ATTENTION = 1,
       SPECA_PROF_FORECAST = 2,  /* Eq. 2: materialised forecast or forecast-and-fold */
       SPECA_PROF_VERIFY = 3,    /* Eq. 4 reductions */
       SPECA_PROF_REFRESH = 4,   /* stand-alone Eq. 3 refresh (the fused one is part of GEMM time) */
       SPECA_PROF_OTHER = 5,     /* conditioning, modulation GEMM, LayerNorm, embed, final layer, solver */
       SPECA_PROF_CLASSES = 6 };

typedef struct speca_profile {
  int64_t launches[SPECA_PROF_CLASSES];
  double  ms[SPECA_PROF_CLASSES];      /* sum of HIP-event durations on the context's stream */
  double  flops[SPECA_PROF_CLASSES];   /* algorithmic: 2 per multiply-add of the contraction */
  double  bytes[SPECA_PROF_CLASSES];   /* algorithmic: tensors the method must read + write once */
} speca_profile;

/* Lanes (an execution option, not part of the method; Sec. 3.2's steps are computed per sample, so
 * the rows of a launch are independent).  A step runs its rows in up to `lanes` groups side by side
 * on library-owned streams forked from and joined to the context's stream with events, so callers
 * see the usual stream order and bit-identical results.  Default 4 (SPECA_LANES in the environment
 * at create overrides), 1 = strictly serial, at most 4.  While a profile is open steps run serially
 * (per-kernel event times are only meaningful without overlap) unless profile_keeps_lanes != 0.
 * Returns SPECA_EINVAL for a value outside 1..4. */
int speca_set_lanes(speca_ctx* ctx, int lanes, int profile_keeps_lanes);

/* While a profile is open every kernel launch of the context is bracketed by a HIP event pair
 * on its stream (this serialises launches and costs a few microseconds each: time a workload
 * for throughput with the profile closed).  speca_profile_end synchronises and sums. */
int speca_profile_begin(speca_ctx* ctx);
int speca_profile_end(speca_ctx* ctx, speca_profile* out);

/* ---- host-only helpers (no device work; usable without a GPU) ----------------------------- */

/* tau[s] = tau0 * beta^(s/S)   (Sec. 3.4.2 adaptive threshold, progress (T-t)/T = s/S). */
int speca_tau_geometric(float tau0, float beta, int steps, float* tau_out);
/* tau[s] = tau_start + (tau_end - tau_start) * s/(S-1). */
int speca_tau_linear(float tau_start, float tau_end, int steps, float* tau_out);
/* Forecast weights c[0..order] for `step` given the references (latest first), k = step - refs[0]:
 *   TAYLOR           c_i = k^i / i!                          (Eq. 2 on differences divided by the last gap)
 *   NEWTON           c_i = prod_{j<i} (step - refs[j])       (backward divided differences)
 *   ADAMS_BASHFORTH  c_0 = 1, c_i = k gamma_{i-1} g^{i-1}    (one explicit Adams step of size k on the slopes
 *                    between references, gamma = 1, 1/2, 5/12, 3/8, g = refs[0] - refs[1]; the draft-model
 *                    ablation of the appendix names this predictor without a formula: textbook coefficients). */
int speca_coefficients(int coef_mode, int step, const int32_t* refs, int n_refs, int order, float* c_out);
/* Refresh divisors d[1..order] written to d_out[0..order-1]. */
int speca_divisors(int coef_mode, int step, const int32_t* refs, int n_refs, int order, float* d_out);

/* RING layout: weights of the stored features in the forecast for `step`, after full steps at
 * full_steps[0..n_full) (increasing) with a cache of order `order`.  w_out[j] multiplies the feature of age j
 * (0 = latest), plane_out[j] is the cache plane that holds it; *n_out = features held (<= order+1).  The
 * weights are sum_i c_i W[i][j], where D^i = sum_j W[i][j] F(age j) follows the refresh recursion of the
 * chosen policy (Eq. 3 with the divisors of speca_divisors). */
int speca_ring_weights(int coef_mode, int order, const int32_t* full_steps, int n_full, int step, float* w_out, int32_t* plane_out,
                       int* n_out);

/* The per-sample schedule state machine of speca_sample, exposed for host-side testing.
 * plan: fills spec_out / full_out (HOST, capacity batch) with the samples to attempt
 * speculatively / to compute in full at `step` under threshold tau_s.
 * commit: accept[i] (HOST) is the verdict for spec list entry i of the last plan; rejected
 * samples and the planned-full ones take `step` as new reference.  kind_out (HOST [batch],
 * may be NULL) receives SPECA_KIND_* of every sample for this step. */
typedef struct speca_sched speca_sched;
int speca_sched_create(speca_sched** out, int batch, const speca_cfg* cfg);
int speca_sched_destroy(speca_sched* s);
int speca_sched_plan(speca_sched* s, int step, float tau_s, int32_t* spec_out, int* n_spec, int32_t* full_out, int* n_full);
int speca_sched_commit(speca_sched* s, int step, const uint8_t* accept, int8_t* kind_out);
/* References of one sample, latest first; returns their count via n_out (<= order+1). */
int speca_sched_refs(const speca_sched* s, int sample, int32_t* refs_out, int* n_out);

#ifdef __cplusplus
}
#endif
#endif /* SPECA_H */
