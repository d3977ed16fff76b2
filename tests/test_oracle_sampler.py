"""Pins of the oracle's sampling loop: schedule rules on scripted models, solver
closed forms, tau=0 => plain sampling, tau=inf => fixed pattern (no GPU)."""
import numpy as np
import pytest

import speca_inputs as si
from oracle import dit, sampler, speca_core as core
from oracle.sampler import KIND_FULL, KIND_SPEC, KIND_REJECT


class ScriptedModel:
    """Two one-slot blocks whose branch output depends only on the conditioning
    timestep: F(t) = script(t) * ones.  Hidden state = x; gates = 1; output = 0.
    Lets a test dictate the verification error at every step."""

    class _S:
        num_classes = 10

    def __init__(self, script):
        self.script = script
        self.n_blocks, self.slots_per_block, self.n_slots = 2, [1, 1], 2
        self.s = self._S()
        self.calls = []

    def begin(self, x, t, labels):
        return np.zeros((len(labels), 1, 4)), t

    def block_real(self, l, h, c):
        self.calls.append(("real", l, c))
        f = np.full_like(h, self.script(c))
        return h + f, [f]

    def block_fold(self, l, h, c, feats):
        return h + feats[0]

    def finish(self, h, c):
        return np.zeros((h.shape[0], 1, 2, 2))

    def forward(self, x, t, labels):
        h, c = self.begin(x, t, labels)
        feats = []
        for l in range(2):
            h, f = self.block_real(l, h, c)
            feats += f
        self.calls.append(("full", c))
        return self.finish(h, c), feats


def _solver(S):
    return sampler.Solver("flow", np.arange(S, dtype=np.float32), np.linspace(1, 0, S + 1).astype(np.float32))


def _run(script, S, tau, **cfg):
    m = ScriptedModel(script)
    out, tr = sampler.sample(m, sampler.SpecaConfig(**cfg), _solver(S), np.asarray(tau, np.float32),
                             np.zeros((1, 1, 2, 2)), [0])
    return m, tr


def test_infinite_threshold_gives_fixed_pattern():
    # linear feature: forecast exact from the second reference on; everything is accepted
    m, tr = _run(lambda t: 2.0 + 0.5 * t, 13, [np.inf] * 13, order=1, interval=4)
    exp = [KIND_FULL if s % 4 == 0 else KIND_SPEC for s in range(13)]
    assert tr.kind[0].tolist() == exp
    assert np.nanmax(tr.err[0, 5:]) < 1e-6          # order-1 forecast of a linear feature is exact
    # first window has one reference only: order 0 reuse, error = |F(0)-F(k)|/F(k)
    assert tr.err[0, 2, 0] == pytest.approx(abs(2.0 - 3.0) / 3.0, rel=1e-6)


def test_zero_threshold_never_speculates():
    m, tr = _run(lambda t: 1.0, 9, [0.0] * 9, order=2, interval=3)
    assert tr.kind[0].tolist() == [KIND_FULL] * 9
    assert np.all(np.isnan(tr.err))
    assert sum(1 for c in m.calls if c[0] == "full") == 9
    assert sum(1 for c in m.calls if c[0] == "real") == 18        # only the full forwards ran blocks


def test_rejection_falls_back_and_rebases():
    # constant feature with a jump at t=6: reuse is exact until the jump, rejected there
    script = lambda t: 1.0 if t < 6 else 3.0
    m, tr = _run(script, 12, [0.1] * 12, order=0, interval=5)
    k = tr.kind[0].tolist()
    # full at 0; 1..4 accepted; 5 forced (5-0 >= N); 6 rejected -> full, new reference; 7..10 accepted; 11 forced
    assert k == [0, 1, 1, 1, 1, 0, 2, 1, 1, 1, 1, 0]
    assert tr.err[0, 6, 0] == pytest.approx(2.0 / 3.0, rel=1e-6)
    assert tr.err[0, 7, 0] == 0.0
    # the rejected step ran the verify block and then a full forward
    full_ts = [c[1] for c in m.calls if c[0] == "full"]
    assert full_ts == [0.0, 5.0, 6.0, 11.0]


def test_accept_is_inclusive_and_uses_step_threshold():
    # reuse error at step s is |1 - (1+0.1 s)|/(1+0.1 s)
    script = lambda t: 1.0 + 0.1 * t
    e = lambda s: np.float32(np.float32(0.1 * s) / np.float32(1 + 0.1 * s))
    S = 4
    errs = [core.relative_error_f32(np.full(4, 1.0), np.full(4, script(float(s)))) for s in range(S)]
    tau = [1.0, float(errs[1]), float(np.nextafter(errs[2], np.float32(0))), 1.0]
    m, tr = _run(script, S, tau, order=0, interval=10)
    # step 1: e == tau -> accepted; step 2: e just above tau -> rejected, becomes reference; step 3: vs new reference
    assert tr.kind[0].tolist() == [0, 1, 2, 1]
    assert tr.err[0, 3, 0] == pytest.approx(0.1 / 1.3, rel=1e-5)


def test_warmup_full_steps():
    _, tr = _run(lambda t: 1.0, 8, [1.0] * 8, order=1, interval=4, warmup_full=3)
    assert tr.kind[0].tolist() == [0, 0, 0, 1, 1, 1, 0, 1]


def test_accepted_steps_do_not_touch_cache():
    # quadratic feature, order 1: if an accepted step refreshed the cache the later errors would change
    script = lambda t: 1.0 + 0.01 * t * t
    _, tr = _run(script, 7, [np.inf] * 7, order=1, interval=100, warmup_full=2)
    # references stay at steps 0 and 1: forecast(s) = F(1) + (s-1)(F(1)-F(0))
    for s in range(2, 7):
        pred = script(1) + (s - 1) * (script(1) - script(0))
        assert tr.err[0, s, 0] == pytest.approx(abs(pred - script(s)) / script(s), rel=1e-5)


def test_cfg_pair_accepts_only_if_both_rows_pass():
    class PairModel(ScriptedModel):
        def block_real(self, l, h, c):
            f = np.zeros_like(h)
            f[0] = 1.0                                    # conditional row: constant -> e = 0
            f[1] = 1.0 if c < 2 else 2.0                  # unconditional row jumps at t=2
            return h + f, [f]
    m = PairModel(None)
    sol = _solver(4); sol.cfg_scale = 1.5
    out, tr = sampler.sample(m, sampler.SpecaConfig(order=0, interval=10), sol, np.full(4, 0.1, np.float32),
                             np.zeros((1, 1, 2, 2)), [0])
    assert tr.kind[0].tolist() == [0, 1, 2, 1]
    assert tr.err[0, 2, 0] == 0.0 and tr.err[0, 2, 1] == pytest.approx(0.5)


def test_other_metrics_decide_the_schedule():
    """The appendix's other error metrics in place of Eq. 4, on scripted features where every metric has a
    hand value: the branch output of a row is (1 + 0.25 [t >= 2]) * (1, 1, 1, 1) up to step 3 (parallel to
    the reused reference: L1 = Linf = L2 = 0.25 / 1.25 = 0.2, cosine distance 0) and changes direction at t = 4
    (reference (1.25,)*4 against (1.25, 1.25, -1.25, -1.25): the hand values are stated where they are asserted)."""
    class DirModel(ScriptedModel):
        def block_real(self, l, h, c):
            f = np.zeros_like(h)
            v = 1.0 if c < 2 else 1.25
            f[...] = v
            if c >= 4:
                f[..., 2:] = -v
            return h + f, [f]
    def run(metric, tau):
        m = DirModel(None)
        _, tr = sampler.sample(m, sampler.SpecaConfig(order=0, interval=10, metric=metric), _solver(6), np.full(6, tau, np.float32),
                               np.zeros((1, 1, 2, 2)), [0])
        return tr
    # t = 1: identical (0 under every metric); t = 2: scaled by 1.25; t = 4: direction change
    for metric in ("l2", "l1", "linf"):
        tr = run(metric, 0.1)
        assert tr.kind[0].tolist() == [0, 1, 2, 1, 2, 1], metric
        assert tr.err[0, 2, 0] == pytest.approx(0.2, rel=1e-6), metric
    # at t = 4 the reference is (1.25,)*4 and the truth (1.25, 1.25, -1.25, -1.25):
    # L2 = sqrt(2 * 2.5^2) / sqrt(4 * 1.25^2) = sqrt(2), L1 = 5 / 5 = 1, Linf = 2.5 / 1.25 = 2
    assert run("l2", 0.1).err[0, 4, 0] == pytest.approx(np.sqrt(2.0), rel=1e-6)
    assert run("l1", 0.1).err[0, 4, 0] == pytest.approx(1.0, rel=1e-6)
    assert run("linf", 0.1).err[0, 4, 0] == pytest.approx(2.0, rel=1e-6)
    # cosine distance ignores the rescaling at t = 2 (accepted: the reference stays (1,)*4) and sees the turn at
    # t = 4: cos = (1.25 + 1.25 - 1.25 - 1.25) / (|p||t|) = 0, distance 1
    tr = run("cosine", 0.1)
    assert tr.kind[0].tolist() == [0, 1, 1, 1, 2, 1]
    assert tr.err[0, 2, 0] == pytest.approx(0.0, abs=1e-7) and tr.err[0, 4, 0] == pytest.approx(1.0, rel=1e-6)
    # the default is Eq. 4
    assert np.array_equal(run("l2", 0.1).err, sampler.sample(DirModel(None), sampler.SpecaConfig(order=0, interval=10), _solver(6),
                                                             np.full(6, 0.1, np.float32), np.zeros((1, 1, 2, 2)), [0])[1].err, equal_nan=True)


# --- solvers -----------------------------------------------------------------------------


def test_ddim_closed_forms():
    x = np.array([2.0, -1.0])
    # zero predicted noise: pure rescale by sqrt(abar_prev/abar_t)
    np.testing.assert_allclose(sampler.ddim_update(x, 0 * x, 0.25, 1.0), x / 0.5)
    # x = sqrt(a) x0 + sqrt(1-a) eps with the true eps: lands on the same (x0, eps) at the next level
    x0, eps = np.array([0.3, -0.7]), np.array([1.1, 0.4])
    a, b = 0.36, 0.81
    xt = np.sqrt(a) * x0 + np.sqrt(1 - a) * eps
    np.testing.assert_allclose(sampler.ddim_update(xt, eps, a, b), np.sqrt(b) * x0 + np.sqrt(1 - b) * eps, rtol=1e-12)
    np.testing.assert_allclose(sampler.ddim_update(xt, eps, a, 1.0), x0, rtol=1e-12)


def test_ddpm_step_pins():
    """Eq. 1.  Pins: a hand-computed value, the Gaussian posterior mean it must equal when the
    predicted noise is the true one, the clean end, and the variance of the draw."""
    # by hand: abar_t = .36, abar_prev = .81 -> alpha = 4/9, beta = 5/9;
    # mu = (1 - (5/9)/0.8 * 0.5) / (2/3) = 0.9791666..., x' = mu + sqrt(5/9) * 1.2 = 1.8735938...
    got = sampler.ddpm_update(np.array([1.0]), np.array([0.5]), 0.36, 0.81, np.array([1.2]))
    np.testing.assert_allclose(got, [0.97916666666666667 + 0.7453559924999299 * 1.2], rtol=1e-14)
    # true noise: the mean is the posterior mean of q(x_prev | x_t, x0)
    x0, eps = np.array([0.3, -0.7, 1.9]), np.array([1.1, 0.4, -0.8])
    a, b = 0.36, 0.81
    al, be = a / b, 1 - a / b
    xt = np.sqrt(a) * x0 + np.sqrt(1 - a) * eps
    post = np.sqrt(b) * be / (1 - a) * x0 + np.sqrt(al) * (1 - b) / (1 - a) * xt
    np.testing.assert_allclose(sampler.ddpm_update(xt, eps, a, b, 0 * xt), post, rtol=1e-13)
    # clean end: abar_prev = 1 returns x0, as the deterministic solver does
    np.testing.assert_allclose(sampler.ddpm_update(xt, eps, a, 1.0, 0 * xt), x0, rtol=1e-13)
    np.testing.assert_allclose(sampler.ddpm_update(xt, eps, a, 1.0, 0 * xt), sampler.ddim_update(xt, eps, a, 1.0), rtol=1e-13)
    # no noise level change: nothing moves
    np.testing.assert_allclose(sampler.ddpm_update(xt, eps, a, a, xt), xt, rtol=1e-15)
    # the draw enters with standard deviation sqrt(beta), not beta
    z = np.random.default_rng(0).standard_normal(200000)
    d = sampler.ddpm_update(np.zeros_like(z), np.zeros_like(z), a, b, z)
    assert abs(d.var() / be - 1) < 0.01 and abs(d.mean()) < 0.01


def test_ddpm_trajectory_uses_each_samples_draws(tiny):
    s, m, _, lat, lab = tiny
    ts, ab = si.ddim_tables(6)
    noise = si.make_solver_noise(6, lat.shape, 0)
    sol = sampler.Solver("ddpm", ts, ab, noise=noise)
    plain = sampler.sample_plain(m, sol, lat, lab)
    out, tr = sampler.sample(m, sampler.SpecaConfig(order=1, interval=3), sol, np.zeros(6, np.float32), lat, lab)
    assert np.array_equal(out, plain)
    # the final step adds no noise; every earlier draw matters, per sample
    n2 = noise.copy(); n2[5] += 1.0
    assert np.array_equal(sampler.sample_plain(m, sampler.Solver("ddpm", ts, ab, noise=n2), lat, lab), plain)
    n3 = noise.copy(); n3[4, 1] += 1.0
    o3 = sampler.sample_plain(m, sampler.Solver("ddpm", ts, ab, noise=n3), lat, lab)
    assert np.array_equal(o3[0], plain[0]) and not np.array_equal(o3[1], plain[1])
    # zero draws: one step of it equals its own mean, and differs from the deterministic solver
    z0 = sampler.sample_plain(m, sampler.Solver("ddpm", ts, ab, noise=0 * noise), lat, lab)
    dd = sampler.sample_plain(m, sampler.Solver("ddim", ts, ab), lat, lab)
    assert np.all(np.isfinite(z0)) and not np.allclose(z0, dd)


def test_flow_and_cfg_closed_forms():
    ts, sig = si.flow_tables(10)
    x = np.array([1.0, 2.0]); v = np.array([0.5, -1.0])
    for s in range(10):
        x = sampler.euler_flow_update(x, v, float(sig[s]), float(sig[s + 1]))
    np.testing.assert_allclose(x, np.array([1.0, 2.0]) - v, rtol=1e-6)      # sigma runs 1 -> 0
    assert sampler.cfg_combine(3.0, 1.0, 1.5) == 4.0 and sampler.cfg_combine(3.0, 1.0, 1.0) == 3.0


def test_ddim_tables():
    ts, ab = si.ddim_tables(50)
    assert ts[0] == 980 and ts[-1] == 0 and len(ab) == 51 and ab[-1] == 1.0
    assert np.all(np.diff(ab) > 0) and ab[-2] == pytest.approx(1 - 1e-4)


# --- tiny DiT, configuration 1 --------------------------------------------------------------


@pytest.fixture(scope="module")
def tiny():
    s = si.dit_tiny()
    m = dit.DiTOracle(s, si.make_dit_weights(s, 0))
    ts, ab = si.ddim_tables(20)
    return s, m, sampler.Solver("ddim", ts, ab), si.make_latents(2, 4, 8, 0), si.make_labels(2, s.num_classes, 0)


def test_tiny_dit_tau_zero_is_plain_sampling(tiny):
    s, m, sol, lat, lab = tiny
    plain = sampler.sample_plain(m, sol, lat, lab)
    out, tr = sampler.sample(m, sampler.SpecaConfig(order=1, interval=4), sol, np.zeros(20, np.float32), lat, lab)
    assert np.array_equal(out, plain)                     # bit-identical
    assert np.all(tr.kind == KIND_FULL)


def test_tiny_dit_default_thresholds_exercise_both_paths(tiny):
    s, m, sol, lat, lab = tiny
    tau = core.tau_linear(0.05, 0.01, 20)
    out, tr = sampler.sample(m, sampler.SpecaConfig(order=1, interval=4), sol, tau, lat, lab)
    assert (tr.kind == KIND_SPEC).sum() > 5 and (tr.kind == KIND_REJECT).sum() > 5
    assert not np.array_equal(tr.kind[0], tr.kind[1])     # sample-adaptive: schedules differ
    # never more than N-1 speculative steps in a row
    for b in range(2):
        run = 0
        for k in tr.kind[b]:
            run = run + 1 if k == KIND_SPEC else 0
            assert run <= 3
    # speculation changes the result a little, not wildly
    plain = sampler.sample_plain(m, sol, lat, lab)
    rel = np.abs(out - plain).max() / np.abs(plain).max()
    assert 0 < rel < 0.2


def test_tiny_dit_guided_runs(tiny):
    s, m, _, lat, lab = tiny
    ts, ab = si.ddim_tables(6)
    sol = sampler.Solver("ddim", ts, ab, cfg_scale=1.5)
    out, tr = sampler.sample(m, sampler.SpecaConfig(order=2, interval=3), sol, np.full(6, 1e9, np.float32), lat, lab)
    assert tr.err.shape == (2, 6, 2) and tr.kind[0].tolist() == [0, 1, 1, 0, 1, 1]
    assert np.all(np.isfinite(out))
