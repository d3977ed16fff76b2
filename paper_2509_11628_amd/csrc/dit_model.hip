// Class-conditional DiT in adaLN-Zero form (Sec. 3.1.2: blocks of attention and MLP in the
// residual form x + AdaLN o f(x)) as the target model of the SpeCa step: the reference
// (full) step with the cache refresh fused into the branch epilogues, and the speculative
// attempt (forecast-and-fold, real verify block, Eq. 4, unconditional finish).
//
//   c      = MLP_t(sinusoid(t)) + y_table[label]
//   h0     = patchify(x) Wp^T + bp + pos
//   block: (shift_a, scale_a, gate_a, shift_m, scale_m, gate_m) = SiLU(c) Wmod^T + bmod
//          F_attn = proj(MHA(LN(h)(1+scale_a)+shift_a))        -> cache slot 2l,   h += gate_a F_attn
//          F_mlp  = fc2(GELU(fc1(LN(h)(1+scale_m)+shift_m)))   -> cache slot 2l+1, h += gate_m F_mlp
//   out    = unpatchify((LN(h)(1+scale_f)+shift_f) Wf^T + bf)
#include <cstring>
#include <map>
#include <string>

#include "dit_kernels.h"
#include "gemm.h"
#include "kernels.h"
#include "mmdit_kernels.h"
#include "model.h"

namespace speca {

namespace {

struct BlockW {
  const void *qkv_w, *qkv_b, *proj_w, *proj_b, *fc1_w, *fc1_b, *fc2_w, *fc2_b;
};

struct DiT final : Model {
  speca_model_desc d{};
  int D = 0, Dm = 0, H = 0, hd = 0, L = 0, T = 0, Kp = 0;
  size_t esz = 4;
  // weights (caller-owned)
  const void *t_w1 = nullptr, *t_b1 = nullptr, *t_w2 = nullptr, *t_b2 = nullptr, *y_table = nullptr;
  const void *patch_w = nullptr, *patch_b = nullptr, *pos = nullptr, *final_w = nullptr, *final_b = nullptr;
  std::vector<BlockW> blk;
  // library-owned: all modulation weights [L*6D + 2D, D] and biases concatenated, so that the
  // modulation of every block (and the final layer) is one GEMM per step
  void* mod_w = nullptr;
  void* mod_b = nullptr;
  int64_t mod_n = 0;                 // L*6D + 2D
  int32_t* gate_off_dev = nullptr;   // [2L][2] offset of each slot's gate inside a modulation row
  // trajectory-level modulation [S][batch_rows][mod_n] (see begin_trajectory)
  float* traj_mod = nullptr;
  void* traj_sc = nullptr;
  size_t traj_cap = 0;
  int traj_S = 0, traj_rows = 0;
  bool traj_on = false;
  // workspace for up to cap_rows rows
  int cap_rows = 0;
  void *emb = nullptr, *t_hid = nullptr, *sc = nullptr, *xn = nullptr, *qkv = nullptr, *att = nullptr, *f1 = nullptr;
  float *temb = nullptr, *mod = nullptr, *h = nullptr, *h2 = nullptr, *feat = nullptr, *tok = nullptr;

  ~DiT() override {
    for (void* p : {mod_w, mod_b, static_cast<void*>(gate_off_dev), static_cast<void*>(traj_mod), traj_sc})
      if (p) (void)hipFree(p);
    free_ws();
  }
  void free_ws() {
    for (void* p : {emb, t_hid, sc, xn, qkv, att, f1, static_cast<void*>(temb), static_cast<void*>(mod), static_cast<void*>(h),
                    static_cast<void*>(h2), static_cast<void*>(feat), static_cast<void*>(tok)})
      if (p) (void)hipFree(p);
    emb = t_hid = sc = xn = qkv = att = f1 = nullptr;
    temb = mod = h = h2 = feat = tok = nullptr;
    cap_rows = 0;
  }

  int n_slots() const override { return 2 * L; }
  int n_blocks() const override { return L; }
  int64_t tokens() const override { return T; }
  int hidden() const override { return D; }
  int64_t latent_elems() const override { return static_cast<int64_t>(d.in_channels) * d.latent_h * d.latent_w; }

  Error prepare(speca_ctx* ctx, int batch_rows) override {
    const int rows = std::min(batch_rows, kMaxRows);
    if (rows <= cap_rows) return ok();
    SPECA_HIP(hipStreamSynchronize(ctx->stream));
    free_ws();
    const size_t R = rows, TT = static_cast<size_t>(T);
    auto alloc = [](void** p, size_t bytes) { return hipMalloc(p, bytes) == hipSuccess; };
    bool good = alloc(&emb, R * d.freq_dim * esz) && alloc(&t_hid, R * D * esz) && alloc(&sc, R * D * esz) &&
                alloc(&xn, R * TT * D * esz) && alloc(&qkv, R * TT * 3 * D * esz) && alloc(&att, R * TT * D * esz) &&
                alloc(&f1, R * TT * Dm * esz) && alloc(reinterpret_cast<void**>(&temb), R * D * 4) &&
                alloc(reinterpret_cast<void**>(&mod), R * mod_n * 4) && alloc(reinterpret_cast<void**>(&h), R * TT * D * 4) &&
                alloc(reinterpret_cast<void**>(&h2), R * TT * D * 4) && alloc(reinterpret_cast<void**>(&feat), R * TT * D * 4) &&
                alloc(reinterpret_cast<void**>(&tok), R * TT * Kp * 4);
    if (!good) {
      (void)hipGetLastError();
      free_ws();
      SPECA_FAIL(SPECA_ENOMEM, "cannot allocate the activation workspace for %d rows", rows);
    }
    cap_rows = rows;
    return ok();
  }

  // SiLU(c) of compact rows 0..n-1 (labels of rows[i]) at timestep t, into sc_out [n][D]
  Error cond_vector(hipStream_t st, float t, const int32_t* labels_per_row, const int32_t* rows, int n, void* sc_out) {
    RowLabels lab{};
    for (int i = 0; i < n; ++i) lab.v[i] = labels_per_row[rows[i]];
    SPECA_TRY(launch_sinusoid(d.dtype, emb, n, d.freq_dim, t, st));
    GemmEpi e1;
    e1.mode = EPI_SILU; e1.bias = t_b1; e1.out = t_hid; e1.ldo = D;
    SPECA_TRY(launch_gemm(d.dtype, emb, d.freq_dim, t_w1, d.freq_dim, n, D, d.freq_dim, e1, st));
    GemmEpi e2;
    e2.mode = EPI_F32; e2.bias = t_b2; e2.out = temb; e2.ldo = D;
    SPECA_TRY(launch_gemm(d.dtype, t_hid, D, t_w2, D, n, D, D, e2, st));
    return launch_cond_sum(d.dtype, temb, y_table, lab, n, D, sc_out, st);
  }

  // conditioning + modulation of all blocks for compact rows 0..n-1 at sampling step `step`
  Error conditioning(speca_ctx* ctx, float t, const int32_t* labels_per_row, int step, const int32_t* rows, int n) {
    hipStream_t st = ctx->stream;
    if (traj_on && step >= 0 && step < traj_S) {
      // inside a trajectory the modulation of this step was computed up front: pick the rows
      ProfScope ps(ctx, SPECA_PROF_OTHER, 0.0, 2.0 * n * mod_n * 4);
      RowLabels idx{};
      for (int i = 0; i < n; ++i) idx.v[i] = rows[i];
      return launch_gather_rows(SPECA_F32, traj_mod + static_cast<int64_t>(step) * traj_rows * mod_n, idx, mod, n, mod_n, st);
    }
    ProfScope ps(ctx, SPECA_PROF_OTHER, 2.0 * n * D * (d.freq_dim + D + static_cast<double>(mod_n)), static_cast<double>(mod_n) * D * esz);
    SPECA_TRY(cond_vector(st, t, labels_per_row, rows, n, sc));
    GemmEpi e3;
    e3.mode = EPI_F32; e3.bias = mod_b; e3.out = mod; e3.ldo = mod_n;
    SPECA_TRY(launch_gemm(d.dtype, sc, D, mod_w, D, n, static_cast<int>(mod_n), D, e3, st));
    return ok();
  }

  Error begin_trajectory(speca_ctx* ctx, const speca_cond*, const int32_t* labels_per_row, const float* timesteps, int S) override {
    hipStream_t st = ctx->stream;
    const int R = ctx->batch_rows;
    const size_t total = static_cast<size_t>(S) * R;
    if (total * mod_n * 4 > (static_cast<size_t>(8) << 30)) return ok();      // too large to be worth holding: per-step path
    if (total > traj_cap) {
      SPECA_HIP(hipStreamSynchronize(st));
      if (traj_mod) (void)hipFree(traj_mod);
      if (traj_sc) (void)hipFree(traj_sc);
      traj_mod = nullptr; traj_sc = nullptr; traj_cap = 0;
      if (hipMalloc(reinterpret_cast<void**>(&traj_mod), total * mod_n * 4) != hipSuccess || hipMalloc(&traj_sc, total * D * esz) != hipSuccess) {
        (void)hipGetLastError();
        if (traj_mod) (void)hipFree(traj_mod);
        traj_mod = nullptr;
        return ok();                                                          // no room: per-step path
      }
      traj_cap = total;
    }
    ProfScope ps(ctx, SPECA_PROF_OTHER, 2.0 * total * D * static_cast<double>(mod_n), static_cast<double>(mod_n) * D * esz + total * mod_n * 4.0);
    std::vector<int32_t> rows(cap_rows);
    for (int s = 0; s < S; ++s)
      for (int r0 = 0; r0 < R; r0 += cap_rows) {
        const int n = std::min(cap_rows, R - r0);
        for (int i = 0; i < n; ++i) rows[i] = r0 + i;
        SPECA_TRY(cond_vector(st, timesteps[s], labels_per_row, rows.data(), n, static_cast<char*>(traj_sc) + (static_cast<size_t>(s) * R + r0) * D * esz));
      }
    GemmEpi e;
    e.mode = EPI_F32; e.bias = mod_b; e.out = traj_mod; e.ldo = mod_n;
    SPECA_TRY(launch_gemm(d.dtype, traj_sc, D, mod_w, D, static_cast<int>(total), static_cast<int>(mod_n), D, e, st));
    traj_S = S; traj_rows = R; traj_on = true;
    return ok();
  }
  void end_trajectory() override { traj_on = false; }

  Error embed(speca_ctx* ctx, const float* x, int x_mod, const int32_t* rows, int n) {
    hipStream_t st = ctx->stream;
    ProfScope ps(ctx, SPECA_PROF_OTHER, 0.0, static_cast<double>(n) * T * D * 4);
    RowLabels xr{};
    for (int i = 0; i < n; ++i) xr.v[i] = rows[i] % x_mod;
    return launch_patch_embed(d.dtype, x, xr, patch_w, patch_b, pos, h, n, d.in_channels, d.latent_h, d.latent_w, d.patch, D, st);
  }

  // A lane works on compact rows [o, o + n) of every workspace buffer, on its own stream.
  struct Lane {
    hipStream_t st;
    int o;
    int shared = 0;     // lanes that run side by side (0: this one alone)
  };
  const float* mod_at(int l, int which, int o = 0) const {
    return mod + static_cast<int64_t>(o) * mod_n + static_cast<int64_t>(l) * 6 * D + static_cast<int64_t>(which) * D;
  }
  template <typename P> P* at(P* base, const Lane& ln, int64_t per_row_bytes) const {
    return reinterpret_cast<P*>(reinterpret_cast<char*>(base) + static_cast<int64_t>(ln.o) * per_row_bytes);
  }

  // attention branch of block l on the lane's rows of hidden state hs (hs = row 0 of the buffer):
  // hs += gate_a * proj(MHA(LNmod(hs)))
  Error attn_branch(speca_ctx* ctx, const Lane& ln, int l, float* hs, int n, const RowTable* refresh_rt) {
    hipStream_t st = ln.st;
    const int64_t M = static_cast<int64_t>(n) * T;
    const double Md = static_cast<double>(M);
    const int64_t TD = static_cast<int64_t>(T) * D;
    float* hl = hs + ln.o * TD;
    void* xn_l = at(static_cast<char*>(xn), ln, TD * esz);
    void* qkv_l = at(static_cast<char*>(qkv), ln, 3 * TD * esz);
    void* att_l = at(static_cast<char*>(att), ln, TD * esz);
    {
      ProfScope ps(ctx, st, SPECA_PROF_OTHER, 0.0, Md * D * (4 + esz));
      SPECA_TRY(launch_ln_modulate(d.dtype, hl, mod_at(l, 0, ln.o), mod_at(l, 1, ln.o), mod_n, xn_l, M, T, D, st));
    }
    GemmEpi e;
    e.mode = EPI_STORE; e.bias = blk[l].qkv_b; e.out = qkv_l; e.ldo = 3 * D; e.shared_chip = ln.shared;
    {
      ProfScope ps(ctx, st, SPECA_PROF_GEMM, 2.0 * Md * 3 * D * D, (Md * 4 * D + 3.0 * D * D) * esz);
      SPECA_TRY(launch_gemm(d.dtype, xn_l, D, blk[l].qkv_w, D, static_cast<int>(M), 3 * D, D, e, st));
    }
    if (refresh_rt) {
      ProfScope ps(ctx, st, SPECA_PROF_REFRESH, 0.0, table_tensors(*refresh_rt) * static_cast<double>(TD) * esz);
      SPECA_TRY(launch_cache_warm(ctx->geom, *refresh_rt, 2 * l, st));
    }
    {
      ProfScope ps(ctx, st, SPECA_PROF_ATTENTION, 4.0 * n * H * static_cast<double>(T) * T * hd, Md * 4 * D * esz);
      SPECA_TRY(launch_attention(d.dtype, qkv_l, att_l, D, n, T, H, hd, st));
    }
    GemmEpi b;
    b.shared_chip = ln.shared;
    b.mode = EPI_BRANCH; b.bias = blk[l].proj_b; b.h = hl; b.ldh = D; b.gate = mod_at(l, 2, ln.o); b.gate_stride = mod_n; b.tokens = T;
    if (refresh_rt) { b.refresh = 1; b.slot = 2 * l; b.g = ctx->geom; b.rt = *refresh_rt; }
    ProfScope ps(ctx, st, SPECA_PROF_GEMM, 2.0 * Md * D * D, (Md * D + 1.0 * D * D) * esz + Md * D * 8);
    SPECA_TRY(launch_gemm(d.dtype, att_l, D, blk[l].proj_w, D, static_cast<int>(M), D, D, b, st));
    return ok();
  }

  // MLP branch of block l on the lane's rows.  truth_out != nullptr (row 0 of the buffer): only materialise
  // F_mlp (fp32) there, no residual, no refresh.
  Error mlp_branch(speca_ctx* ctx, const Lane& ln, int l, float* hs, int n, const RowTable* refresh_rt, float* truth_out) {
    hipStream_t st = ln.st;
    const int64_t M = static_cast<int64_t>(n) * T;
    const double Md = static_cast<double>(M);
    const int64_t TD = static_cast<int64_t>(T) * D;
    float* hl = hs + ln.o * TD;
    void* xn_l = at(static_cast<char*>(xn), ln, TD * esz);
    void* f1_l = at(static_cast<char*>(f1), ln, static_cast<int64_t>(T) * Dm * esz);
    {
      ProfScope ps(ctx, st, SPECA_PROF_OTHER, 0.0, Md * D * (4 + esz));
      SPECA_TRY(launch_ln_modulate(d.dtype, hl, mod_at(l, 3, ln.o), mod_at(l, 4, ln.o), mod_n, xn_l, M, T, D, st));
    }
    if (refresh_rt && !truth_out) {
      ProfScope ps(ctx, st, SPECA_PROF_REFRESH, 0.0, table_tensors(*refresh_rt) * static_cast<double>(TD) * esz);
      SPECA_TRY(launch_cache_warm(ctx->geom, *refresh_rt, 2 * l + 1, st));
    }
    GemmEpi e;
    e.mode = EPI_GELU; e.bias = blk[l].fc1_b; e.out = f1_l; e.ldo = Dm; e.shared_chip = ln.shared;
    {
      ProfScope ps(ctx, st, SPECA_PROF_GEMM, 2.0 * Md * Dm * D, (Md * (D + Dm) + 1.0 * D * Dm) * esz);
      SPECA_TRY(launch_gemm(d.dtype, xn_l, D, blk[l].fc1_w, D, static_cast<int>(M), Dm, D, e, st));
    }
    GemmEpi b;
    b.bias = blk[l].fc2_b;
    b.shared_chip = ln.shared;
    if (truth_out) {
      b.mode = EPI_F32; b.out = truth_out + ln.o * TD; b.ldo = D;
    } else {
      b.mode = EPI_BRANCH; b.h = hl; b.ldh = D; b.gate = mod_at(l, 5, ln.o); b.gate_stride = mod_n; b.tokens = T;
      if (refresh_rt) { b.refresh = 1; b.slot = 2 * l + 1; b.g = ctx->geom; b.rt = *refresh_rt; }
    }
    ProfScope ps(ctx, st, SPECA_PROF_GEMM, 2.0 * Md * Dm * D, (Md * Dm + 1.0 * D * Dm) * esz + Md * D * 8);
    SPECA_TRY(launch_gemm(d.dtype, f1_l, Dm, blk[l].fc2_w, Dm, static_cast<int>(M), D, Dm, b, st));
    return ok();
  }

  // Blocks [l0, l1) for all n rows, the row groups of the split side by side (launches interleaved
  // block by block so the lanes stay in step).  refresh_rt / truth as in the branch functions.
  Error run_blocks(speca_ctx* ctx, int l0, int l1, float* hs, int n, const RowTable* refresh_rt, float* truth_last_mlp) {
    // Row groups side by side pay off for whole batches: 16 rows in four groups of four run a reference step 7 % faster
    // than serially.  Eight rows (half a batch recomputed after rejections) are faster as one launch sequence whose tiles
    // are chosen for the whole chip (+7 % on a trajectory of split steps), and the single verify block of a
    // speculative attempt is best in two groups (+1 %).
    const int min_rows = n <= 8 ? n + 1 : (l1 - l0 == 1 ? 8 : 4);
    const LaneSplit ls = split_lanes(ctx, n, min_rows);
    RowTable sub[kMaxLanes];
    if (refresh_rt)
      for (int k = 0; k < ls.n_lanes; ++k) sub[k] = slice_table(*refresh_rt, ls.first[k], ls.first[k + 1] - ls.first[k]);
    SPECA_TRY(lanes_fork(ctx, ls));
    Error body = [&]() -> Error {
      for (int l = l0; l < l1; ++l) {
        for (int k = 0; k < ls.n_lanes; ++k) {
          const Lane ln{ctx->lane_stream[k], ls.first[k], ls.n_lanes > 1 ? ls.n_lanes : 0};
          SPECA_TRY(attn_branch(ctx, ln, l, hs, ls.first[k + 1] - ls.first[k], refresh_rt ? &sub[k] : nullptr));
        }
        for (int k = 0; k < ls.n_lanes; ++k) {
          const Lane ln{ctx->lane_stream[k], ls.first[k], ls.n_lanes > 1 ? ls.n_lanes : 0};
          SPECA_TRY(mlp_branch(ctx, ln, l, hs, ls.first[k + 1] - ls.first[k], refresh_rt ? &sub[k] : nullptr,
                               l == l1 - 1 ? truth_last_mlp : nullptr));
        }
      }
      return ok();
    }();
    Error joined = lanes_join(ctx, ls);        // also after a failed launch: the main stream never runs ahead of a lane
    return body.code != SPECA_OK ? body : joined;
  }

  Error final_layer(speca_ctx* ctx, const float* hs, const int32_t* rows, int n, float* model_out) {
    hipStream_t st = ctx->stream;
    const int64_t M = static_cast<int64_t>(n) * T;
    const float* fm = mod + static_cast<int64_t>(L) * 6 * D;
    ProfScope ps(ctx, SPECA_PROF_OTHER, 2.0 * M * Kp * D, static_cast<double>(M) * D * (4 + 2 * esz));
    SPECA_TRY(launch_ln_modulate(d.dtype, hs, fm, fm + D, mod_n, xn, M, T, D, st));
    GemmEpi e;
    e.mode = EPI_F32; e.bias = final_b; e.out = tok; e.ldo = Kp;
    SPECA_TRY(launch_gemm(d.dtype, xn, D, final_w, D, static_cast<int>(M), Kp, D, e, st));
    RowLabels r{};
    for (int i = 0; i < n; ++i) r.v[i] = rows[i];
    return launch_unpatchify(tok, r, model_out, n, d.in_channels, d.latent_h, d.latent_w, d.patch, st);
  }

  Error full_step(speca_ctx* ctx, const float* x, int x_mod, const speca_cond* cond, const int32_t* labels_per_row, int step,
                  const int32_t* rows, int n, float* model_out) override {
    if (n > cap_rows) SPECA_FAIL(SPECA_EUNSUPPORTED, "at most %d rows per launch", cap_rows);
    RowTable rt;
    SPECA_TRY(build_refresh_table(ctx, step, rows, n, &rt));
    SPECA_TRY(conditioning(ctx, cond->timestep, labels_per_row, step, rows, n));
    SPECA_TRY(embed(ctx, x, x_mod, rows, n));
    SPECA_TRY(run_blocks(ctx, 0, L, h, n, &rt, nullptr));
    SPECA_TRY(final_layer(ctx, h, rows, n, model_out));
    push_refs(ctx, step, rows, n);
    return ok();
  }

  Error spec_step(speca_ctx* ctx, const float* x, int x_mod, const speca_cond* cond, const int32_t* labels_per_row, int step,
                  const int32_t* rows, int n, const float* tau_per_row, int pair_stride, float* model_out) override {
    if (n > cap_rows) SPECA_FAIL(SPECA_EUNSUPPORTED, "at most %d rows per launch", cap_rows);
    hipStream_t st = ctx->stream;
    RowTable rt;
    SPECA_TRY(build_forecast_table(ctx, step, rows, n, &rt));
    // pairs: partner of rows[i] must be listed
    std::vector<int> partner(n, -1);
    if (pair_stride > 0) {
      std::map<int, int> where;
      for (int i = 0; i < n; ++i) where[rows[i]] = i;
      for (int i = 0; i < n; ++i) {
        const int other = rows[i] < pair_stride ? rows[i] + pair_stride : rows[i] - pair_stride;
        auto it = where.find(other);
        if (it == where.end()) SPECA_FAIL(SPECA_EINVAL, "row %d is listed without its pair row %d", rows[i], other);
        partner[i] = it->second;
      }
    }
    const int lv = ctx->cfg.verify_block >= 0 ? ctx->cfg.verify_block : L - 1;
    SPECA_TRY(conditioning(ctx, cond->timestep, labels_per_row, step, rows, n));
    SPECA_TRY(embed(ctx, x, x_mod, rows, n));
    // Eq. 2 for every slot before the verify block, folded into h
    const double tens = table_tensors(rt), Ed = static_cast<double>(ctx->geom.E);
    // and the accepted path's forecasts for the verify block and everything after it -> h2.  One pass over the cache
    // when the verify block sits in the last quarter of the stack (the verify block then waits for a few more slots
    // but the hidden state is read once and there is one launch); two passes otherwise, so that an early verify
    // block does not wait for the whole cache.
    if (4 * lv >= 3 * L) {
      ProfScope ps(ctx, SPECA_PROF_FORECAST, 0.0, 2.0 * L * tens * Ed * esz + 3.0 * n * Ed * 4);
      SPECA_TRY(launch_forecast_fold2(ctx->geom, rt, h, h, 2 * lv, h2, mod, mod_n, gate_off_dev, 0, 0, 2 * L, D, st));
    } else {
      {
        ProfScope ps(ctx, SPECA_PROF_FORECAST, 0.0, 2.0 * lv * tens * Ed * esz + 2.0 * n * Ed * 4);
        SPECA_TRY(launch_forecast_fold(ctx->geom, rt, h, h, mod, mod_n, gate_off_dev, 0, 0, 2 * lv, D, st));
      }
      ProfScope ps(ctx, SPECA_PROF_FORECAST, 0.0, 2.0 * (L - lv) * tens * Ed * esz + 2.0 * n * Ed * 4);
      SPECA_TRY(launch_forecast_fold(ctx->geom, rt, h, h2, mod, mod_n, gate_off_dev, 0, 2 * lv, 2 * L, D, st));
    }
    // the verify block for real, on h
    SPECA_TRY(run_blocks(ctx, lv, lv + 1, h, n, nullptr, feat));
    // Eq. 4: forecast of slot 2lv+1 (formed on the fly from the cache) vs the recomputed feature
    VerifyScratch& v = ctx->vs;
    SPECA_TRY(ensure_partial(ctx, static_cast<size_t>(n) * verify_chunks(ctx->geom.E) * 3));
    std::memcpy(v.h_tau, tau_per_row, n * sizeof(float));
    SPECA_HIP(hipMemcpyAsync(v.tau_dev, v.h_tau, n * sizeof(float), hipMemcpyHostToDevice, st));
    {
      ProfScope ps(ctx, SPECA_PROF_VERIFY, 0.0, tens * Ed * esz + n * Ed * 4);
      SPECA_TRY(launch_verify(ctx->cfg.metric, nullptr, ctx->geom.dtype, feat, SPECA_F32, ctx->geom.E, &ctx->geom, &rt, 2 * lv + 1, n,
                              ctx->cfg.eps, v.tau_dev, v.partial, v.err_dev, v.acc_dev, st));
    }
    SPECA_HIP(hipMemcpyAsync(v.h_err, v.err_dev, n * sizeof(float), hipMemcpyDeviceToHost, st));
    SPECA_HIP(hipMemcpyAsync(v.h_acc, v.acc_dev, n, hipMemcpyDeviceToHost, st));
    // finish every listed row from h2 while the verdict travels; rejected rows are overwritten by the fallback
    SPECA_TRY(final_layer(ctx, h2, rows, n, model_out));
    SPECA_HIP(hipStreamSynchronize(st));
    if (pair_stride > 0) {
      std::vector<uint8_t> both(n);
      for (int i = 0; i < n; ++i) both[i] = v.h_acc[i] && v.h_acc[partner[i]];
      for (int i = 0; i < n; ++i) v.h_acc[i] = both[i];
    }
    return ok();
  }
};

struct WeightLookup {
  std::map<std::string, std::pair<const void*, int64_t>> tab;
  Error get(const std::string& name, int64_t numel, const void** out) const {
    auto it = tab.find(name);
    if (it == tab.end()) SPECA_FAIL(SPECA_EINVAL, "weight '%s' is missing", name.c_str());
    if (!it->second.first) SPECA_FAIL(SPECA_EINVAL, "weight '%s' is NULL", name.c_str());
    if (it->second.second != numel)
      SPECA_FAIL(SPECA_EINVAL, "weight '%s' has %lld elements, expected %lld", name.c_str(), static_cast<long long>(it->second.second),
                 static_cast<long long>(numel));
    *out = it->second.first;
    return ok();
  }
};

}  // namespace

Error make_dit_model(const speca_model_desc& d, const speca_weights* w, std::unique_ptr<Model>* out) {
  if (!w || w->count < 1 || !w->names || !w->ptrs || !w->numel) SPECA_FAIL(SPECA_EINVAL, "a DiT context needs a weight table");
  if (d.depth < 1 || d.heads < 1 || d.hidden % d.heads) SPECA_FAIL(SPECA_EINVAL, "depth/heads/hidden = %d/%d/%d", d.depth, d.heads, d.hidden);
  if (d.patch < 1 || d.latent_h % d.patch || d.latent_w % d.patch || d.latent_h < 1 || d.latent_w < 1)
    SPECA_FAIL(SPECA_EINVAL, "latent %dx%d is not a multiple of patch %d", d.latent_h, d.latent_w, d.patch);
  if (d.latent_t != 1) SPECA_FAIL(SPECA_EINVAL, "DiT takes image latents (latent_t = 1)");
  if (d.in_channels < 1 || d.mlp_hidden < 1 || d.num_classes < 1 || d.freq_dim < 2 || d.freq_dim % 2)
    SPECA_FAIL(SPECA_EINVAL, "in_channels/mlp_hidden/num_classes/freq_dim invalid");
  std::unique_ptr<DiT> m(new DiT());
  m->d = d;
  m->D = d.hidden; m->Dm = d.mlp_hidden; m->H = d.heads; m->hd = d.hidden / d.heads; m->L = d.depth;
  m->T = (d.latent_h / d.patch) * (d.latent_w / d.patch);
  m->Kp = d.in_channels * d.patch * d.patch;
  m->esz = dtype_size(d.dtype);
  if (m->D % 8 || m->Dm % 8 || m->Kp % 4 || d.freq_dim % 8)
    SPECA_FAIL(SPECA_EUNSUPPORTED, "hidden, mlp_hidden, freq_dim must be multiples of 8 and C*p*p of 4");
  const int64_t D = m->D, Dm = m->Dm;
  WeightLookup wl;
  for (int i = 0; i < w->count; ++i) wl.tab[w->names[i] ? w->names[i] : ""] = {w->ptrs[i], w->numel[i]};
  SPECA_TRY(wl.get("t_w1", D * d.freq_dim, &m->t_w1));
  SPECA_TRY(wl.get("t_b1", D, &m->t_b1));
  SPECA_TRY(wl.get("t_w2", D * D, &m->t_w2));
  SPECA_TRY(wl.get("t_b2", D, &m->t_b2));
  SPECA_TRY(wl.get("y_table", (d.num_classes + 1) * D, &m->y_table));
  SPECA_TRY(wl.get("patch_w", D * m->Kp, &m->patch_w));
  SPECA_TRY(wl.get("patch_b", D, &m->patch_b));
  SPECA_TRY(wl.get("pos", static_cast<int64_t>(m->T) * D, &m->pos));
  SPECA_TRY(wl.get("final_w", static_cast<int64_t>(m->Kp) * D, &m->final_w));
  SPECA_TRY(wl.get("final_b", m->Kp, &m->final_b));
  m->blk.resize(m->L);
  m->mod_n = static_cast<int64_t>(m->L) * 6 * D + 2 * D;
  SPECA_HIP(hipMalloc(&m->mod_w, static_cast<size_t>(m->mod_n) * D * m->esz));
  SPECA_HIP(hipMalloc(&m->mod_b, static_cast<size_t>(m->mod_n) * m->esz));
  for (int l = 0; l < m->L; ++l) {
    const std::string p = "blk" + std::to_string(l) + ".";
    BlockW& b = m->blk[l];
    SPECA_TRY(wl.get(p + "qkv_w", 3 * D * D, &b.qkv_w));
    SPECA_TRY(wl.get(p + "qkv_b", 3 * D, &b.qkv_b));
    SPECA_TRY(wl.get(p + "proj_w", D * D, &b.proj_w));
    SPECA_TRY(wl.get(p + "proj_b", D, &b.proj_b));
    SPECA_TRY(wl.get(p + "fc1_w", Dm * D, &b.fc1_w));
    SPECA_TRY(wl.get(p + "fc1_b", Dm, &b.fc1_b));
    SPECA_TRY(wl.get(p + "fc2_w", D * Dm, &b.fc2_w));
    SPECA_TRY(wl.get(p + "fc2_b", D, &b.fc2_b));
    const void *mw, *mb;
    SPECA_TRY(wl.get(p + "mod_w", 6 * D * D, &mw));
    SPECA_TRY(wl.get(p + "mod_b", 6 * D, &mb));
    SPECA_HIP(hipMemcpy(static_cast<char*>(m->mod_w) + static_cast<size_t>(l) * 6 * D * D * m->esz, mw, 6 * D * D * m->esz, hipMemcpyDeviceToDevice));
    SPECA_HIP(hipMemcpy(static_cast<char*>(m->mod_b) + static_cast<size_t>(l) * 6 * D * m->esz, mb, 6 * D * m->esz, hipMemcpyDeviceToDevice));
  }
  const void *fw, *fb;
  SPECA_TRY(wl.get("fmod_w", 2 * D * D, &fw));
  SPECA_TRY(wl.get("fmod_b", 2 * D, &fb));
  SPECA_HIP(hipMemcpy(static_cast<char*>(m->mod_w) + static_cast<size_t>(m->L) * 6 * D * D * m->esz, fw, 2 * D * D * m->esz, hipMemcpyDeviceToDevice));
  SPECA_HIP(hipMemcpy(static_cast<char*>(m->mod_b) + static_cast<size_t>(m->L) * 6 * D * m->esz, fb, 2 * D * m->esz, hipMemcpyDeviceToDevice));
  std::vector<int32_t> goff(4 * m->L);          // [slot][2]: one stream, both entries equal
  for (int l = 0; l < m->L; ++l) {
    goff[4 * l] = goff[4 * l + 1] = static_cast<int32_t>((static_cast<int64_t>(l) * 6 + 2) * D);
    goff[4 * l + 2] = goff[4 * l + 3] = static_cast<int32_t>((static_cast<int64_t>(l) * 6 + 5) * D);
  }
  SPECA_HIP(hipMalloc(reinterpret_cast<void**>(&m->gate_off_dev), goff.size() * sizeof(int32_t)));
  SPECA_HIP(hipMemcpy(m->gate_off_dev, goff.data(), goff.size() * sizeof(int32_t), hipMemcpyHostToDevice));
  SPECA_HIP(hipDeviceSynchronize());
  out->reset(m.release());
  return ok();
}

}  // namespace speca
