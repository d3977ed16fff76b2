// Rectified-flow MMDiT (dual-stream blocks with joint attention over [text ; image] tokens,
// then single-stream blocks; rotary positions; per-head RMS-norm on q and k) as the second
// target-model family of the SpeCa step (the paper's FLUX and HunyuanVideo workloads,
// Sec. 4 / appendix "Model Configurations"; the block definition is this library's own).
//
//   vec = MLP_t(sinusoid(t)) + MLP_v(pooled);  h = [txt_in(text) ; img_in(patchify(x))]
//   dual block l (stream s in {txt, img}, own weights, own 6-way modulation):
//       qkv_s = LNmod(h_s) Wqkv_s;  q,k <- RoPE(RMSnorm(q,k));  a = joint attention
//       F_attn = [a_txt Wproj_txt ; a_img Wproj_img]   -> cache slot 2l      h += gate_a(s) F_attn
//       F_mlp  = [mlp_txt(LNmod(h_txt)) ; mlp_img(..)] -> cache slot 2l+1    h += gate_m(s) F_mlp
//   single block l (3-way modulation):
//       [qkv | m] = LNmod(h) W1;  a = attention(RoPE(RMSnorm(q,k)), v)
//       F = [a | GELU(m)] W2                           -> cache slot 2*n_dual + l   h += gate F
//   out = unpatchify(LNmod(h_img) Wf)
// Cached slots are joint over the [text ; image] token sequence, so every slot has the same
// geometry [rows][Tt + Ti][D]; the gates differ per stream only.
#include <cstring>
#include <map>
#include <string>

#include "gemm.h"
#include "kernels.h"
#include "mmdit_kernels.h"
#include "model.h"

namespace speca {

namespace {

struct StreamW {
  const void *qkv_w, *qkv_b, *qnorm, *knorm, *proj_w, *proj_b, *fc1_w, *fc1_b, *fc2_w, *fc2_b;
};
struct SingleW {
  const void *lin1_w, *lin1_b, *qnorm, *knorm, *lin2_w, *lin2_b;
};

struct MMDiT final : Model {
  speca_model_desc d{};
  int D = 0, Dm = 0, H = 0, hd = 0, nd = 0, ns = 0, Tt = 0, Ti = 0, T = 0, Kp = 0;
  size_t esz = 4;
  const void *t_w1 = nullptr, *t_b1 = nullptr, *t_w2 = nullptr, *t_b2 = nullptr, *v_w1 = nullptr, *v_b1 = nullptr, *v_w2 = nullptr,
             *v_b2 = nullptr, *img_in_w = nullptr, *img_in_b = nullptr, *txt_in_w = nullptr, *txt_in_b = nullptr, *final_w = nullptr,
             *final_b = nullptr;
  const float *rope_cos = nullptr, *rope_sin = nullptr;
  std::vector<StreamW> img, txt;      // per dual block
  std::vector<SingleW> single;
  void *mod_w = nullptr, *mod_b = nullptr;
  int64_t mod_n = 0, base_s = 0, base_f = 0;
  int32_t* gate_off_dev = nullptr;    // [n_slots][2]
  std::vector<int> first_slot;        // per block, plus end
  float* traj_mod = nullptr;          // [S][batch_rows][mod_n], see begin_trajectory
  void* traj_sc = nullptr;
  size_t traj_cap = 0;
  int traj_S = 0, traj_rows = 0;
  bool traj_on = false;
  int cap_rows = 0;
  void *emb = nullptr, *t_hid = nullptr, *v_in = nullptr, *v_hid = nullptr, *sc = nullptr, *patches = nullptr, *xn = nullptr, *qkv = nullptr,
       *att = nullptr, *f1 = nullptr, *cat = nullptr;
  float *temb = nullptr, *vemb = nullptr, *mod = nullptr, *h = nullptr, *h2 = nullptr, *feat = nullptr, *tok = nullptr;

  ~MMDiT() override {
    for (void* p : {mod_w, mod_b, static_cast<void*>(gate_off_dev), static_cast<void*>(traj_mod), traj_sc})
      if (p) (void)hipFree(p);
    free_ws();
  }
  void free_ws() {
    void* all[] = {emb, t_hid, v_in, v_hid, sc, patches, xn, qkv, att, f1, cat, temb, vemb, mod, h, h2, feat, tok};
    for (void* p : all)
      if (p) (void)hipFree(p);
    emb = t_hid = v_in = v_hid = sc = patches = xn = qkv = att = f1 = cat = nullptr;
    temb = vemb = mod = h = h2 = feat = tok = nullptr;
    cap_rows = 0;
  }

  int n_slots() const override { return 2 * nd + ns; }
  int n_blocks() const override { return nd + ns; }
  int64_t tokens() const override { return T; }
  int hidden() const override { return D; }
  int64_t latent_elems() const override { return static_cast<int64_t>(d.in_channels) * d.latent_t * d.latent_h * d.latent_w; }

  Error prepare(speca_ctx* ctx, int batch_rows) override {
    const int rows = std::min(batch_rows, kMaxRows);
    if (rows <= cap_rows) return ok();
    SPECA_HIP(hipStreamSynchronize(ctx->stream));
    free_ws();
    const size_t R = rows, TT = static_cast<size_t>(T);
    auto al = [](auto** p, size_t bytes) { return hipMalloc(reinterpret_cast<void**>(p), bytes) == hipSuccess; };
    const bool good = al(&emb, R * d.freq_dim * esz) && al(&t_hid, R * D * esz) && al(&v_in, R * d.vec_dim * esz) && al(&v_hid, R * D * esz) &&
                      al(&sc, R * D * esz) && al(&patches, R * Ti * Kp * esz) && al(&xn, R * TT * D * esz) && al(&qkv, R * TT * 3 * D * esz) &&
                      al(&att, R * TT * D * esz) && al(&f1, R * TT * Dm * esz) && al(&cat, R * TT * (D + Dm) * esz) && al(&temb, R * D * 4) &&
                      al(&vemb, R * D * 4) && al(&mod, R * mod_n * 4) && al(&h, R * TT * D * 4) && al(&h2, R * TT * D * 4) &&
                      al(&feat, R * TT * D * 4) && al(&tok, R * Ti * Kp * 4);
    if (!good) {
      (void)hipGetLastError();
      free_ws();
      SPECA_FAIL(SPECA_ENOMEM, "cannot allocate the activation workspace for %d rows", rows);
    }
    cap_rows = rows;
    return ok();
  }

  Error gemm(speca_ctx* ctx, int cls, const void* A, int64_t lda, const void* W, int64_t ldw, int64_t M, int N, int K, const GemmEpi& e) {
    ProfScope ps(ctx, cls, 2.0 * M * N * K, (static_cast<double>(M) * (K + N) + static_cast<double>(N) * K) * esz);
    return launch_gemm(d.dtype, A, lda, W, ldw, static_cast<int>(M), N, K, e, ctx->stream);
  }

  // SiLU(vec) of compact rows 0..n-1 at timestep t, into sc_out [n][D]
  Error cond_vector(speca_ctx* ctx, float t, const speca_cond* cond, const int32_t* rows, int n, void* sc_out) {
    hipStream_t st = ctx->stream;
    if (!cond->pooled) SPECA_FAIL(SPECA_EINVAL, "cond->pooled is NULL");
    SPECA_TRY(launch_sinusoid(d.dtype, emb, n, d.freq_dim, t, st));
    GemmEpi e;
    e.mode = EPI_SILU; e.bias = t_b1; e.out = t_hid; e.ldo = D;
    SPECA_TRY(launch_gemm(d.dtype, emb, d.freq_dim, t_w1, d.freq_dim, n, D, d.freq_dim, e, st));
    e = GemmEpi(); e.mode = EPI_F32; e.bias = t_b2; e.out = temb; e.ldo = D;
    SPECA_TRY(launch_gemm(d.dtype, t_hid, D, t_w2, D, n, D, D, e, st));
    RowLabels idx{};
    for (int i = 0; i < n; ++i) idx.v[i] = rows[i];
    SPECA_TRY(launch_gather_rows(d.dtype, cond->pooled, idx, v_in, n, d.vec_dim, st));
    e = GemmEpi(); e.mode = EPI_SILU; e.bias = v_b1; e.out = v_hid; e.ldo = D;
    SPECA_TRY(launch_gemm(d.dtype, v_in, d.vec_dim, v_w1, d.vec_dim, n, D, d.vec_dim, e, st));
    e = GemmEpi(); e.mode = EPI_F32; e.bias = v_b2; e.out = vemb; e.ldo = D;
    SPECA_TRY(launch_gemm(d.dtype, v_hid, D, v_w2, D, n, D, D, e, st));
    return launch_silu_sum(d.dtype, temb, vemb, sc_out, static_cast<int64_t>(n) * D, st);
  }

  Error conditioning(speca_ctx* ctx, const speca_cond* cond, int step, const int32_t* rows, int n) {
    hipStream_t st = ctx->stream;
    if (traj_on && step >= 0 && step < traj_S) {
      ProfScope ps(ctx, SPECA_PROF_OTHER, 0.0, 2.0 * n * mod_n * 4);
      RowLabels idx{};
      for (int i = 0; i < n; ++i) idx.v[i] = rows[i];
      return launch_gather_rows(SPECA_F32, traj_mod + static_cast<int64_t>(step) * traj_rows * mod_n, idx, mod, n, mod_n, st);
    }
    ProfScope ps(ctx, SPECA_PROF_OTHER, 2.0 * n * D * static_cast<double>(mod_n), static_cast<double>(mod_n) * D * esz);
    SPECA_TRY(cond_vector(ctx, cond->timestep, cond, rows, n, sc));
    GemmEpi e;
    e.mode = EPI_F32; e.bias = mod_b; e.out = mod; e.ldo = mod_n;
    return launch_gemm(d.dtype, sc, D, mod_w, D, n, static_cast<int>(mod_n), D, e, st);
  }

  Error begin_trajectory(speca_ctx* ctx, const speca_cond* cond, const int32_t*, const float* timesteps, int S) override {
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
        return ok();
      }
      traj_cap = total;
    }
    ProfScope ps(ctx, SPECA_PROF_OTHER, 2.0 * total * D * static_cast<double>(mod_n), static_cast<double>(mod_n) * D * esz + total * mod_n * 4.0);
    std::vector<int32_t> rows(cap_rows);
    for (int s = 0; s < S; ++s)
      for (int r0 = 0; r0 < R; r0 += cap_rows) {
        const int n = std::min(cap_rows, R - r0);
        for (int i = 0; i < n; ++i) rows[i] = r0 + i;
        SPECA_TRY(cond_vector(ctx, timesteps[s], cond, rows.data(), n, static_cast<char*>(traj_sc) + (static_cast<size_t>(s) * R + r0) * D * esz));
      }
    GemmEpi e;
    e.mode = EPI_F32; e.bias = mod_b; e.out = traj_mod; e.ldo = mod_n;
    SPECA_TRY(launch_gemm(d.dtype, traj_sc, D, mod_w, D, static_cast<int>(total), static_cast<int>(mod_n), D, e, st));
    traj_S = S; traj_rows = R; traj_on = true;
    return ok();
  }
  void end_trajectory() override { traj_on = false; }

  Error embed(speca_ctx* ctx, const float* x, int x_mod, const speca_cond* cond, const int32_t* rows, int n) {
    hipStream_t st = ctx->stream;
    if (!cond->txt) SPECA_FAIL(SPECA_EINVAL, "cond->txt is NULL");
    RowLabels xr{};
    for (int i = 0; i < n; ++i) xr.v[i] = rows[i] % x_mod;
    SPECA_TRY(launch_patchify(d.dtype, x, xr, patches, n, d.in_channels, d.latent_t, d.latent_h, d.latent_w, d.patch, st));
    for (int i = 0; i < n; ++i) {
      GemmEpi e;
      e.mode = EPI_F32; e.bias = txt_in_b; e.out = h + static_cast<int64_t>(i) * T * D; e.ldo = D;
      const char* a = static_cast<const char*>(cond->txt) + static_cast<size_t>(rows[i]) * Tt * d.txt_dim * esz;
      SPECA_TRY(gemm(ctx, SPECA_PROF_OTHER, a, d.txt_dim, txt_in_w, d.txt_dim, Tt, D, d.txt_dim, e));
      e.bias = img_in_b; e.out = h + (static_cast<int64_t>(i) * T + Tt) * D;
      const char* pa = static_cast<const char*>(patches) + static_cast<size_t>(i) * Ti * Kp * esz;
      SPECA_TRY(gemm(ctx, SPECA_PROF_OTHER, pa, Kp, img_in_w, Kp, Ti, D, Kp, e));
    }
    return ok();
  }

  const char* at(const void* p, int64_t elems) const { return static_cast<const char*>(p) + elems * esz; }
  char* at(void* p, int64_t elems) const { return static_cast<char*>(p) + elems * esz; }

  Error attention_part(speca_ctx* ctx, int n, const void* qn_t, const void* kn_t, const void* qn_i, const void* kn_i, void* out, int64_t ldo) {
    hipStream_t st = ctx->stream;
    const double Md = static_cast<double>(n) * T;
    {
      ProfScope ps(ctx, SPECA_PROF_OTHER, 0.0, Md * 2 * D * esz * 2);
      SPECA_TRY(launch_qk_norm_rope(d.dtype, qkv, 3 * D, static_cast<int64_t>(n) * T, T, Tt, H, hd, qn_t, kn_t, qn_i, kn_i, rope_cos, rope_sin, st));
    }
    ProfScope ps(ctx, SPECA_PROF_ATTENTION, 4.0 * n * H * static_cast<double>(T) * T * hd, Md * 4 * D * esz);
    return launch_attention(d.dtype, qkv, out, ldo, n, T, H, hd, st);
  }

  // One single-row table out of a multi-row one.
  static RowTable one_row(const RowTable& rt, int i) {
    RowTable r{};
    r.n = 1;
    r.row[0] = rt.row[i];
    r.order[0] = rt.order[i];
    for (int o = 0; o < kMaxTensors; ++o) r.w[0][o] = rt.w[i][o];
    return r;
  }

  // Dual block l on hidden state hs.  refresh_rt: refresh cache slots 2l, 2l+1.  truth_out: materialise
  // the MLP slot (fp32) there instead of folding it (verification).
  Error dual_block(speca_ctx* ctx, int l, float* hs, int n, const RowTable* refresh_rt, float* truth_out) {
    hipStream_t st = ctx->stream;
    const int64_t NT = static_cast<int64_t>(n) * T;
    const float* mi = mod + static_cast<int64_t>(l) * 12 * D;      // image modulation: shift_a, scale_a, gate_a, shift_m, scale_m, gate_m
    const float* mt = mi + 6 * D;                                   // text modulation
    const StreamW* sw[2] = {&txt[l], &img[l]};
    const float* sm[2] = {mt, mi};
    const int off[2] = {0, Tt}, len[2] = {Tt, Ti};
    {
      ProfScope ps(ctx, SPECA_PROF_OTHER, 0.0, static_cast<double>(NT) * D * (4 + esz));
      SPECA_TRY(launch_ln_modulate2(d.dtype, hs, mt, mt + D, mi, mi + D, Tt, mod_n, xn, NT, T, D, st));
    }
    for (int i = 0; i < n; ++i)
      for (int s = 0; s < 2; ++s) {
        const int64_t t0 = static_cast<int64_t>(i) * T + off[s];
        GemmEpi e;
        e.mode = EPI_STORE; e.bias = sw[s]->qkv_b; e.out = at(qkv, t0 * 3 * D); e.ldo = 3 * D;
        SPECA_TRY(gemm(ctx, SPECA_PROF_GEMM, at(xn, t0 * D), D, sw[s]->qkv_w, D, len[s], 3 * D, D, e));
      }
    SPECA_TRY(attention_part(ctx, n, txt[l].qnorm, txt[l].knorm, img[l].qnorm, img[l].knorm, att, D));
    for (int i = 0; i < n; ++i)
      for (int s = 0; s < 2; ++s) {
        const int64_t t0 = static_cast<int64_t>(i) * T + off[s];
        GemmEpi b;
        b.mode = EPI_BRANCH; b.bias = sw[s]->proj_b; b.h = hs + t0 * D; b.ldh = D; b.gate = sm[s] + 2 * D + static_cast<int64_t>(i) * mod_n;
        b.gate_stride = 0; b.tokens = len[s];
        if (refresh_rt) { b.refresh = 1; b.slot = 2 * l; b.g = ctx->geom; b.rt = one_row(*refresh_rt, i); b.cache_elem_offset = static_cast<int64_t>(off[s]) * D; }
        SPECA_TRY(gemm(ctx, SPECA_PROF_GEMM, at(att, t0 * D), D, sw[s]->proj_w, D, len[s], D, D, b));
      }
    {
      ProfScope ps(ctx, SPECA_PROF_OTHER, 0.0, static_cast<double>(NT) * D * (4 + esz));
      SPECA_TRY(launch_ln_modulate2(d.dtype, hs, mt + 3 * D, mt + 4 * D, mi + 3 * D, mi + 4 * D, Tt, mod_n, xn, NT, T, D, st));
    }
    for (int i = 0; i < n; ++i)
      for (int s = 0; s < 2; ++s) {
        const int64_t t0 = static_cast<int64_t>(i) * T + off[s];
        GemmEpi e;
        e.mode = EPI_GELU; e.bias = sw[s]->fc1_b; e.out = at(f1, t0 * Dm); e.ldo = Dm;
        SPECA_TRY(gemm(ctx, SPECA_PROF_GEMM, at(xn, t0 * D), D, sw[s]->fc1_w, D, len[s], Dm, D, e));
        GemmEpi b;
        b.bias = sw[s]->fc2_b;
        if (truth_out) {
          b.mode = EPI_F32; b.out = truth_out + t0 * D; b.ldo = D;
        } else {
          b.mode = EPI_BRANCH; b.h = hs + t0 * D; b.ldh = D; b.gate = sm[s] + 5 * D + static_cast<int64_t>(i) * mod_n; b.gate_stride = 0;
          b.tokens = len[s];
          if (refresh_rt) { b.refresh = 1; b.slot = 2 * l + 1; b.g = ctx->geom; b.rt = one_row(*refresh_rt, i); b.cache_elem_offset = static_cast<int64_t>(off[s]) * D; }
        }
        SPECA_TRY(gemm(ctx, SPECA_PROF_GEMM, at(f1, t0 * Dm), Dm, sw[s]->fc2_w, Dm, len[s], D, Dm, b));
      }
    return ok();
  }

  Error single_block(speca_ctx* ctx, int l, float* hs, int n, const RowTable* refresh_rt, float* truth_out) {
    hipStream_t st = ctx->stream;
    const int64_t NT = static_cast<int64_t>(n) * T;
    const float* ms = mod + base_s + static_cast<int64_t>(l) * 3 * D;     // shift, scale, gate
    const SingleW& w = single[l];
    const int Dc = D + Dm;
    {
      ProfScope ps(ctx, SPECA_PROF_OTHER, 0.0, static_cast<double>(NT) * D * (4 + esz));
      SPECA_TRY(launch_ln_modulate(d.dtype, hs, ms, ms + D, mod_n, xn, NT, T, D, st));
    }
    GemmEpi e;
    e.mode = EPI_STORE; e.bias = w.lin1_b; e.out = qkv; e.ldo = 3 * D;
    SPECA_TRY(gemm(ctx, SPECA_PROF_GEMM, xn, D, w.lin1_w, D, NT, 3 * D, D, e));
    e = GemmEpi(); e.mode = EPI_GELU; e.bias = at(w.lin1_b, 3 * D); e.out = at(cat, D); e.ldo = Dc;
    SPECA_TRY(gemm(ctx, SPECA_PROF_GEMM, xn, D, at(w.lin1_w, static_cast<int64_t>(3) * D * D), D, NT, Dm, D, e));
    SPECA_TRY(attention_part(ctx, n, w.qnorm, w.knorm, w.qnorm, w.knorm, cat, Dc));
    GemmEpi b;
    b.bias = w.lin2_b;
    if (truth_out) {
      b.mode = EPI_F32; b.out = truth_out; b.ldo = D;
    } else {
      b.mode = EPI_BRANCH; b.h = hs; b.ldh = D; b.gate = ms + 2 * D; b.gate_stride = mod_n; b.tokens = T;
      if (refresh_rt) { b.refresh = 1; b.slot = 2 * nd + l; b.g = ctx->geom; b.rt = *refresh_rt; }
    }
    SPECA_TRY(gemm(ctx, SPECA_PROF_GEMM, cat, Dc, w.lin2_w, Dc, NT, D, Dc, b));
    return ok();
  }

  Error block(speca_ctx* ctx, int b, float* hs, int n, const RowTable* refresh_rt, float* truth_out) {
    return b < nd ? dual_block(ctx, b, hs, n, refresh_rt, truth_out) : single_block(ctx, b - nd, hs, n, refresh_rt, truth_out);
  }

  Error final_layer(speca_ctx* ctx, const float* hs, const int32_t* rows, int n, float* model_out) {
    hipStream_t st = ctx->stream;
    const float* fm = mod + base_f;
    ProfScope ps(ctx, SPECA_PROF_OTHER, 2.0 * n * Ti * Kp * D, static_cast<double>(n) * Ti * D * (4 + 2 * esz));
    for (int i = 0; i < n; ++i)
      SPECA_TRY(launch_ln_modulate(d.dtype, hs + (static_cast<int64_t>(i) * T + Tt) * D, fm + static_cast<int64_t>(i) * mod_n,
                                   fm + D + static_cast<int64_t>(i) * mod_n, mod_n, at(xn, static_cast<int64_t>(i) * Ti * D), Ti, Ti, D, st));
    GemmEpi e;
    e.mode = EPI_F32; e.bias = final_b; e.out = tok; e.ldo = Kp;
    SPECA_TRY(launch_gemm(d.dtype, xn, D, final_w, D, n * Ti, Kp, D, e, st));
    RowLabels r{};
    for (int i = 0; i < n; ++i) r.v[i] = rows[i];
    return launch_unpatchify_video(tok, r, model_out, n, d.in_channels, d.latent_t, d.latent_h, d.latent_w, d.patch, st);
  }

  Error begin(speca_ctx* ctx, const float* x, int x_mod, const speca_cond* cond, int step, const int32_t* rows, int n) {
    SPECA_TRY(conditioning(ctx, cond, step, rows, n));
    return embed(ctx, x, x_mod, cond, rows, n);
  }

  Error full_step(speca_ctx* ctx, const float* x, int x_mod, const speca_cond* cond, const int32_t*, int step, const int32_t* rows, int n,
                  float* model_out) override {
    if (n > cap_rows) SPECA_FAIL(SPECA_EUNSUPPORTED, "at most %d rows per launch", cap_rows);
    RowTable rt;
    SPECA_TRY(build_refresh_table(ctx, step, rows, n, &rt));
    SPECA_TRY(begin(ctx, x, x_mod, cond, step, rows, n));
    for (int b = 0; b < nd + ns; ++b) SPECA_TRY(block(ctx, b, h, n, &rt, nullptr));
    SPECA_TRY(final_layer(ctx, h, rows, n, model_out));
    push_refs(ctx, step, rows, n);
    return ok();
  }

  Error spec_step(speca_ctx* ctx, const float* x, int x_mod, const speca_cond* cond, const int32_t*, int step, const int32_t* rows, int n,
                  const float* tau_per_row, int pair_stride, float* model_out) override {
    if (n > cap_rows) SPECA_FAIL(SPECA_EUNSUPPORTED, "at most %d rows per launch", cap_rows);
    if (pair_stride != 0) SPECA_FAIL(SPECA_EUNSUPPORTED, "guidance pairs are not part of the rectified-flow models");
    hipStream_t st = ctx->stream;
    RowTable rt;
    SPECA_TRY(build_forecast_table(ctx, step, rows, n, &rt));
    const int nb = nd + ns;
    const int lv = ctx->cfg.verify_block >= 0 ? ctx->cfg.verify_block : nb - 1;
    const int s_lv = first_slot[lv], s_end = first_slot[nb], v_slot = first_slot[lv + 1] - 1;
    SPECA_TRY(begin(ctx, x, x_mod, cond, step, rows, n));
    const double tens = table_tensors(rt), Ed = static_cast<double>(ctx->geom.E);
    const int64_t split = static_cast<int64_t>(Tt) * D;
    // one pass over the cache for both hidden states when the verify block sits in the last quarter of the stack
    if (4 * lv >= 3 * nb) {
      ProfScope ps(ctx, SPECA_PROF_FORECAST, 0.0, s_end * tens * Ed * esz + 3.0 * n * Ed * 4);
      SPECA_TRY(launch_forecast_fold2(ctx->geom, rt, h, h, s_lv, h2, mod, mod_n, gate_off_dev, split, 0, s_end, D, st));
    } else {
      {
        ProfScope ps(ctx, SPECA_PROF_FORECAST, 0.0, s_lv * tens * Ed * esz + 2.0 * n * Ed * 4);
        SPECA_TRY(launch_forecast_fold(ctx->geom, rt, h, h, mod, mod_n, gate_off_dev, split, 0, s_lv, D, st));
      }
      ProfScope ps(ctx, SPECA_PROF_FORECAST, 0.0, (s_end - s_lv) * tens * Ed * esz + 2.0 * n * Ed * 4);
      SPECA_TRY(launch_forecast_fold(ctx->geom, rt, h, h2, mod, mod_n, gate_off_dev, split, s_lv, s_end, D, st));
    }
    SPECA_TRY(block(ctx, lv, h, n, nullptr, feat));
    VerifyScratch& v = ctx->vs;
    SPECA_TRY(ensure_partial(ctx, static_cast<size_t>(n) * verify_chunks(ctx->geom.E) * 3));
    std::memcpy(v.h_tau, tau_per_row, n * sizeof(float));
    SPECA_HIP(hipMemcpyAsync(v.tau_dev, v.h_tau, n * sizeof(float), hipMemcpyHostToDevice, st));
    {
      ProfScope ps(ctx, SPECA_PROF_VERIFY, 0.0, tens * Ed * esz + n * Ed * 4);
      SPECA_TRY(launch_verify(ctx->cfg.metric, nullptr, ctx->geom.dtype, feat, SPECA_F32, ctx->geom.E, &ctx->geom, &rt, v_slot, n, ctx->cfg.eps,
                              v.tau_dev, v.partial, v.err_dev, v.acc_dev, st));
    }
    SPECA_HIP(hipMemcpyAsync(v.h_err, v.err_dev, n * sizeof(float), hipMemcpyDeviceToHost, st));
    SPECA_HIP(hipMemcpyAsync(v.h_acc, v.acc_dev, n, hipMemcpyDeviceToHost, st));
    SPECA_TRY(final_layer(ctx, h2, rows, n, model_out));
    SPECA_HIP(hipStreamSynchronize(st));
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

Error make_mmdit_model(const speca_model_desc& d, const speca_weights* w, std::unique_ptr<Model>* out) {
  if (!w || w->count < 1 || !w->names || !w->ptrs || !w->numel) SPECA_FAIL(SPECA_EINVAL, "an MMDiT context needs a weight table");
  if (d.depth < 0 || d.depth_single < 0 || d.depth + d.depth_single < 1) SPECA_FAIL(SPECA_EINVAL, "depth/depth_single = %d/%d", d.depth, d.depth_single);
  if (d.heads < 1 || d.hidden % d.heads) SPECA_FAIL(SPECA_EINVAL, "heads/hidden = %d/%d", d.heads, d.hidden);
  if (d.patch < 1 || d.latent_t < 1 || d.latent_h < 1 || d.latent_w < 1 || d.latent_h % d.patch || d.latent_w % d.patch)
    SPECA_FAIL(SPECA_EINVAL, "latent %dx%dx%d / patch %d", d.latent_t, d.latent_h, d.latent_w, d.patch);
  if (d.txt_tokens < 1 || d.txt_dim < 1 || d.vec_dim < 1 || d.in_channels < 1 || d.mlp_hidden < 1 || d.freq_dim < 2 || d.freq_dim % 2)
    SPECA_FAIL(SPECA_EINVAL, "txt_tokens/txt_dim/vec_dim/in_channels/mlp_hidden/freq_dim invalid");
  std::unique_ptr<MMDiT> m(new MMDiT());
  m->d = d;
  m->D = d.hidden; m->Dm = d.mlp_hidden; m->H = d.heads; m->hd = d.hidden / d.heads; m->nd = d.depth; m->ns = d.depth_single;
  m->Tt = d.txt_tokens; m->Ti = d.latent_t * (d.latent_h / d.patch) * (d.latent_w / d.patch); m->T = m->Tt + m->Ti;
  m->Kp = d.in_channels * d.patch * d.patch;
  m->esz = dtype_size(d.dtype);
  if (m->D % 8 || m->Dm % 8 || m->Kp % 4 || d.freq_dim % 8 || d.txt_dim % 8 || d.vec_dim % 8 || m->hd % 2 || m->hd > 128)
    SPECA_FAIL(SPECA_EUNSUPPORTED, "hidden, mlp_hidden, freq_dim, txt_dim, vec_dim must be multiples of 8, C*p*p of 4, head_dim even and <= 128");
  const int64_t D = m->D, Dm = m->Dm, hd = m->hd;
  WeightLookup wl;
  for (int i = 0; i < w->count; ++i) wl.tab[w->names[i] ? w->names[i] : ""] = {w->ptrs[i], w->numel[i]};
  SPECA_TRY(wl.get("t_w1", D * d.freq_dim, &m->t_w1));
  SPECA_TRY(wl.get("t_b1", D, &m->t_b1));
  SPECA_TRY(wl.get("t_w2", D * D, &m->t_w2));
  SPECA_TRY(wl.get("t_b2", D, &m->t_b2));
  SPECA_TRY(wl.get("v_w1", D * d.vec_dim, &m->v_w1));
  SPECA_TRY(wl.get("v_b1", D, &m->v_b1));
  SPECA_TRY(wl.get("v_w2", D * D, &m->v_w2));
  SPECA_TRY(wl.get("v_b2", D, &m->v_b2));
  SPECA_TRY(wl.get("img_in_w", D * m->Kp, &m->img_in_w));
  SPECA_TRY(wl.get("img_in_b", D, &m->img_in_b));
  SPECA_TRY(wl.get("txt_in_w", D * d.txt_dim, &m->txt_in_w));
  SPECA_TRY(wl.get("txt_in_b", D, &m->txt_in_b));
  SPECA_TRY(wl.get("final_w", static_cast<int64_t>(m->Kp) * D, &m->final_w));
  SPECA_TRY(wl.get("final_b", m->Kp, &m->final_b));
  const void *rc, *rs;
  SPECA_TRY(wl.get("rope_cos", static_cast<int64_t>(m->T) * (hd / 2), &rc));
  SPECA_TRY(wl.get("rope_sin", static_cast<int64_t>(m->T) * (hd / 2), &rs));
  m->rope_cos = static_cast<const float*>(rc);
  m->rope_sin = static_cast<const float*>(rs);
  m->base_s = static_cast<int64_t>(m->nd) * 12 * D;
  m->base_f = m->base_s + static_cast<int64_t>(m->ns) * 3 * D;
  m->mod_n = m->base_f + 2 * D;
  SPECA_HIP(hipMalloc(&m->mod_w, static_cast<size_t>(m->mod_n) * D * m->esz));
  SPECA_HIP(hipMalloc(&m->mod_b, static_cast<size_t>(m->mod_n) * m->esz));
  auto put = [&](int64_t row0, int64_t nrows, const void* mw, const void* mb) -> Error {
    SPECA_HIP(hipMemcpy(static_cast<char*>(m->mod_w) + static_cast<size_t>(row0) * D * m->esz, mw, static_cast<size_t>(nrows) * D * m->esz, hipMemcpyDeviceToDevice));
    SPECA_HIP(hipMemcpy(static_cast<char*>(m->mod_b) + static_cast<size_t>(row0) * m->esz, mb, static_cast<size_t>(nrows) * m->esz, hipMemcpyDeviceToDevice));
    return ok();
  };
  m->img.resize(m->nd);
  m->txt.resize(m->nd);
  for (int l = 0; l < m->nd; ++l)
    for (int s = 0; s < 2; ++s) {
      const std::string p = "dual" + std::to_string(l) + (s == 0 ? ".img_" : ".txt_");
      StreamW& sw = s == 0 ? m->img[l] : m->txt[l];
      SPECA_TRY(wl.get(p + "qkv_w", 3 * D * D, &sw.qkv_w));
      SPECA_TRY(wl.get(p + "qkv_b", 3 * D, &sw.qkv_b));
      SPECA_TRY(wl.get(p + "qnorm", hd, &sw.qnorm));
      SPECA_TRY(wl.get(p + "knorm", hd, &sw.knorm));
      SPECA_TRY(wl.get(p + "proj_w", D * D, &sw.proj_w));
      SPECA_TRY(wl.get(p + "proj_b", D, &sw.proj_b));
      SPECA_TRY(wl.get(p + "fc1_w", Dm * D, &sw.fc1_w));
      SPECA_TRY(wl.get(p + "fc1_b", Dm, &sw.fc1_b));
      SPECA_TRY(wl.get(p + "fc2_w", D * Dm, &sw.fc2_w));
      SPECA_TRY(wl.get(p + "fc2_b", D, &sw.fc2_b));
      const void *mw, *mb;
      SPECA_TRY(wl.get(p + "mod_w", 6 * D * D, &mw));
      SPECA_TRY(wl.get(p + "mod_b", 6 * D, &mb));
      SPECA_TRY(put(static_cast<int64_t>(l) * 12 * D + (s == 0 ? 0 : 6 * D), 6 * D, mw, mb));
    }
  m->single.resize(m->ns);
  for (int l = 0; l < m->ns; ++l) {
    const std::string p = "single" + std::to_string(l) + ".";
    SingleW& sw = m->single[l];
    SPECA_TRY(wl.get(p + "lin1_w", (3 * D + Dm) * D, &sw.lin1_w));
    SPECA_TRY(wl.get(p + "lin1_b", 3 * D + Dm, &sw.lin1_b));
    SPECA_TRY(wl.get(p + "qnorm", hd, &sw.qnorm));
    SPECA_TRY(wl.get(p + "knorm", hd, &sw.knorm));
    SPECA_TRY(wl.get(p + "lin2_w", D * (D + Dm), &sw.lin2_w));
    SPECA_TRY(wl.get(p + "lin2_b", D, &sw.lin2_b));
    const void *mw, *mb;
    SPECA_TRY(wl.get(p + "mod_w", 3 * D * D, &mw));
    SPECA_TRY(wl.get(p + "mod_b", 3 * D, &mb));
    SPECA_TRY(put(m->base_s + static_cast<int64_t>(l) * 3 * D, 3 * D, mw, mb));
  }
  const void *fw, *fb;
  SPECA_TRY(wl.get("fmod_w", 2 * D * D, &fw));
  SPECA_TRY(wl.get("fmod_b", 2 * D, &fb));
  SPECA_TRY(put(m->base_f, 2 * D, fw, fb));
  if (m->mod_n > 0x7FFFFFFF) SPECA_FAIL(SPECA_EUNSUPPORTED, "modulation row too wide");
  // gate offsets [slot][2] = (text, image) and the slot map
  std::vector<int32_t> goff(2 * (2 * m->nd + m->ns));
  m->first_slot.clear();
  for (int l = 0; l < m->nd; ++l) {
    m->first_slot.push_back(2 * l);
    const int64_t bi = static_cast<int64_t>(l) * 12 * D, bt = bi + 6 * D;
    goff[2 * (2 * l) + 0] = static_cast<int32_t>(bt + 2 * D);
    goff[2 * (2 * l) + 1] = static_cast<int32_t>(bi + 2 * D);
    goff[2 * (2 * l + 1) + 0] = static_cast<int32_t>(bt + 5 * D);
    goff[2 * (2 * l + 1) + 1] = static_cast<int32_t>(bi + 5 * D);
  }
  for (int l = 0; l < m->ns; ++l) {
    m->first_slot.push_back(2 * m->nd + l);
    const int32_t g = static_cast<int32_t>(m->base_s + static_cast<int64_t>(l) * 3 * D + 2 * D);
    goff[2 * (2 * m->nd + l)] = goff[2 * (2 * m->nd + l) + 1] = g;
  }
  m->first_slot.push_back(2 * m->nd + m->ns);
  SPECA_HIP(hipMalloc(reinterpret_cast<void**>(&m->gate_off_dev), goff.size() * sizeof(int32_t)));
  SPECA_HIP(hipMemcpy(m->gate_off_dev, goff.data(), goff.size() * sizeof(int32_t), hipMemcpyHostToDevice));
  SPECA_HIP(hipDeviceSynchronize());
  out->reset(m.release());
  return ok();
}

}  // namespace speca
