"""CPU oracle of the SpeCa sampling loop (forecast -> verify -> accept / fall back).

TEST INFRASTRUCTURE ONLY (see oracle/speca_core.py).

Follows Sec. 3.2 (three-step workflow), Sec. 3.3 (Eq. 2-3), Sec. 3.4 (Eq. 4,
sequential validation, adaptive threshold).  Samples are independent: each has
its own cache, reference history and accept/reject path (the paper's
sample-adaptive allocation), so the loop below simply runs sample by sample.

Readings (paper silent / ambiguous):
  * a full step is forced when s - r0 >= N (N = forced activation period), so at
    most N-1 consecutive speculative steps follow a full step;
  * a rejected step is itself recomputed in full and becomes the new reference;
  * tau[s] <= 0 schedules step s as full without speculating (threshold 0
    reproduces plain sampling exactly);
  * the verified tensor is the last cached slot of the verify block, recomputed
    for real from the hidden state propagated with forecasts; the error is taken
    over all tokens x channels of one batch row;
  * an accepted step uses forecasts for every block, the verify block included,
    and leaves the cache untouched;
  * with classifier-free guidance a sample is two rows (conditional,
    unconditional); it is accepted iff both rows pass.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

from . import speca_core as core

KIND_FULL = 0          # scheduled full step
KIND_SPEC = 1          # speculative step, accepted
KIND_REJECT = 2        # speculative attempt rejected -> recomputed in full


# ----------------------------------------------------------------------------- solvers


def ddim_update(x, eps, abar_t, abar_prev):
    """Deterministic DDIM (eta = 0): x0 = (x - sqrt(1-abar_t) eps)/sqrt(abar_t);
    x' = sqrt(abar_prev) x0 + sqrt(1-abar_prev) eps."""
    x0 = (x - np.sqrt(1.0 - abar_t) * eps) / np.sqrt(abar_t)
    return np.sqrt(abar_prev) * x0 + np.sqrt(1.0 - abar_prev) * eps


def euler_flow_update(x, v, sigma_t, sigma_next):
    """Rectified-flow Euler step: x' = x + (sigma_next - sigma_t) v."""
    return x + (sigma_next - sigma_t) * v


def ddpm_update(x, eps, abar_t, abar_prev, z):
    """One ancestral sampling step, Eq. 1: x' ~ N(mu, beta I) with
    mu = (x - (1 - alpha) / sqrt(1 - abar_t) eps) / sqrt(alpha).
    On a sub-sampled schedule the per-step alpha is the ratio of the two cumulative products,
    alpha = abar_t / abar_prev, and beta = 1 - alpha (reading: the paper does not spell out the
    respacing).  `z` is the standard-normal draw, passed in; the caller passes zeros at the final
    step, which returns the mean (reading: the usual convention, the paper is silent)."""
    alpha = abar_t / abar_prev
    beta = 1.0 - alpha
    mu = (x - beta / np.sqrt(1.0 - abar_t) * eps) / np.sqrt(alpha)
    return mu + np.sqrt(beta) * z


def cfg_combine(out_cond, out_uncond, scale):
    return out_uncond + scale * (out_cond - out_uncond)


@dataclass
class Solver:
    kind: str                 # "ddim" | "flow" | "ddpm"
    timesteps: np.ndarray     # [S] value the model is conditioned on at step s
    table: np.ndarray         # [S+1] alpha_bar (ddim, ddpm) or sigma (flow)
    cfg_scale: float = 0.0    # > 0: classifier-free guidance with an extra null-label row
    noise: Optional[np.ndarray] = None   # ddpm: [S, B, *latent] standard-normal draws (step S-1 is not used)

    @property
    def steps(self) -> int:
        return len(self.timesteps)

    def update(self, x, out, s, sample=0):
        a, b = float(self.table[s]), float(self.table[s + 1])
        if self.kind == "ddim":
            return ddim_update(x, out, a, b)
        if self.kind == "flow":
            return euler_flow_update(x, out, a, b)
        if self.kind == "ddpm":
            z = np.zeros_like(x) if s == self.steps - 1 else np.asarray(self.noise[s][sample], np.float64).reshape(x.shape)
            return ddpm_update(x, out, a, b, z)
        raise ValueError(self.kind)


@dataclass
class SpecaConfig:
    order: int = 2                 # m
    interval: int = 5              # N
    verify_block: int = -1         # -1 = last block
    mode: str = "taylor"           # coefficient policy
    eps: float = core.EPS_DEFAULT
    warmup_full: int = 1           # steps 0..warmup_full-1 are always full
    cache_store: Optional[str] = None   # None (float64) | "f32" | "bf16": storage rounding of the cache
    cache_layout: str = "differences"   # "differences" (Sec. 3.3 as described) | "ring" (raw features, same forecasts)
    metric: str = "l2"             # "l2" (Eq. 4) | "l1" | "linf" | "cosine" (appendix "Choice of Error Metrics")


@dataclass
class Trace:
    kind: np.ndarray     # [B, S] int8
    err: np.ndarray      # [B, S, rows_per_sample] float32 (nan where not verified)
    tau: np.ndarray      # [S] float32

    @property
    def n_full(self):
        return int(np.sum(self.kind != KIND_SPEC))

    @property
    def alpha(self):
        return float(np.mean(self.kind == KIND_SPEC))


# ----------------------------------------------------------------------------- one sample


def _rows_for_sample(model, solver: Solver, cond):
    """Conditioning of the rows of one sample.  Class-conditional models: `cond` is the label;
    with guidance a second row carries the null label.  Models with their own `rows_cond`
    (text-conditioned) take `cond` as is."""
    if hasattr(model, "rows_cond"):
        return model.rows_cond(cond, solver.cfg_scale > 0)
    if solver.cfg_scale > 0:
        return [int(cond), int(model.s.num_classes)]       # conditional row, null-label row
    return [int(cond)]


def _model_out(out_rows, solver: Solver):
    if solver.cfg_scale > 0:
        return cfg_combine(out_rows[0], out_rows[1], solver.cfg_scale)
    return out_rows[0]


def full_step(model, cache: core.FeatureCache, x_rows, t, labels, s):
    """Step 1 of the workflow: complete forward, cache refresh."""
    out, feats = model.forward(x_rows, t, labels)
    cache.refresh(s, feats)
    return out


def verification_error(metric: str, pred, truth, eps: float) -> np.float32:
    """The error the verifier compares with the threshold, rounded to float32 (the precision of the decision).
    Eq. 4 by default; the other metrics of the appendix ablation on request."""
    if metric == "l2":
        return core.relative_error_f32(pred, truth, eps)
    fn = {"l1": core.relative_error_l1, "linf": core.relative_error_linf, "cosine": core.cosine_distance}[metric]
    return np.float32(fn(pred, truth, eps))


def speculative_attempt(model, cache: core.FeatureCache, cfg: SpecaConfig, x_rows, t, labels, s, tau_s):
    """Steps 2-3 of the workflow for one sample at step s.
    -> (accepted, per-row errors, model output rows or None)."""
    lv = cfg.verify_block if cfg.verify_block >= 0 else model.n_blocks - 1
    first_slot = [0]
    for n in model.slots_per_block:
        first_slot.append(first_slot[-1] + n)
    Fp = [cache.forecast(s, j) for j in range(model.n_slots)]           # Eq. 2, every slot
    h, c = model.begin(x_rows, t, labels)
    for l in range(lv):                                                # blocks before the verify block
        h = model.block_fold(l, h, c, Fp[first_slot[l]:first_slot[l + 1]])
    _, real = model.block_real(lv, h, c)                               # the verify block, for real
    v = first_slot[lv + 1] - 1                                         # last slot of the verify block
    Ft = real[-1]
    errs = [verification_error(cfg.metric, Fp[v][r], Ft[r], cfg.eps) for r in range(Ft.shape[0])]   # Eq. 4 per row
    ok = all(core.accept(e, tau_s) for e in errs)
    if not ok:
        return False, errs, None
    for l in range(lv, model.n_blocks):                                # accepted: forecasts everywhere
        h = model.block_fold(l, h, c, Fp[first_slot[l]:first_slot[l + 1]])
    return True, errs, model.finish(h, c)


def sample_one(model, cfg: SpecaConfig, solver: Solver, tau: np.ndarray, x0: np.ndarray, label, sample_index: int = 0):
    """Whole trajectory of one sample.  x0: [C,(T,)H,W].  -> (final latent, kinds[S], errs[S,rows]).
    sample_index picks the sample's draws out of solver.noise (stochastic solver only)."""
    S = solver.steps
    labels = _rows_for_sample(model, solver, label)
    R = 2 if solver.cfg_scale > 0 else 1
    cache = core.make_cache(cfg.cache_layout, model.n_slots, cfg.order, cfg.mode, cfg.cache_store)
    x = np.asarray(x0, dtype=np.float64)
    kinds = np.zeros(S, dtype=np.int8)
    errs = np.full((S, R), np.nan, dtype=np.float32)
    for s in range(S):
        t = float(solver.timesteps[s])
        x_rows = np.repeat(x[None], R, axis=0)
        spec = (len(cache.refs) >= 1 and (s - cache.refs[0]) < cfg.interval
                and s >= cfg.warmup_full and float(tau[s]) > 0.0)
        out_rows = None
        if spec:
            ok, e, out_rows = speculative_attempt(model, cache, cfg, x_rows, t, labels, s, tau[s])
            errs[s] = e
            kinds[s] = KIND_SPEC if ok else KIND_REJECT
            spec = ok
        if not spec:
            out_rows = full_step(model, cache, x_rows, t, labels, s)
        x = solver.update(x, _model_out(out_rows, solver), s, sample_index)
    return x, kinds, errs


def sample(model, cfg: SpecaConfig, solver: Solver, tau: np.ndarray, latents: np.ndarray, labels: Sequence[int]):
    """SpeCa sampling of a batch.  -> (final latents [B,C,H,W] float64, Trace)."""
    B = latents.shape[0]
    S = solver.steps
    R = 2 if solver.cfg_scale > 0 else 1
    out = np.empty(latents.shape, dtype=np.float64)
    tr = Trace(np.zeros((B, S), np.int8), np.full((B, S, R), np.nan, np.float32), np.asarray(tau, np.float32))
    for b in range(B):
        out[b], tr.kind[b], tr.err[b] = sample_one(model, cfg, solver, tr.tau, latents[b], labels[b], b)
    return out, tr


def sample_plain(model, solver: Solver, latents: np.ndarray, labels: Sequence[int]):
    """Ordinary sampling: a full forward at every step, no cache."""
    B = latents.shape[0]
    out = np.empty(latents.shape, dtype=np.float64)
    for b in range(B):
        x = np.asarray(latents[b], dtype=np.float64)
        lab = _rows_for_sample(model, solver, labels[b])
        R = 2 if solver.cfg_scale > 0 else 1
        for s in range(solver.steps):
            o, _ = model.forward(np.repeat(x[None], R, axis=0), float(solver.timesteps[s]), lab)
            x = solver.update(x, _model_out(o, solver), s, b)
        out[b] = x
    return out
