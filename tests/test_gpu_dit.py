"""Parity of the DiT reference step, the speculative attempt and the whole SpeCa
trajectory with the CPU oracle, through the C ABI.

Bars: accept/reject decisions and schedules equal (both sides take the decision in
fp32 on the same fp32 thresholds; the smallest relative margin |e - tau| / tau is
printed so that a decision inside rounding noise would be visible);
final latents max-abs error / max-abs value <= 1e-5 for fp32 models and <= 2e-2 for
bf16 models."""
import numpy as np
import pytest

import speca_inputs as si
from oracle import dit as odit, sampler as osamp, speca_core as core

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def max_abs_rel(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-30))


def make_gpu(shape, weights):
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    dt = bd.BF16 if shape.dtype == "bf16" else bd.F32
    return sp.Context(sp.dit_desc(shape), sp.to_device(weights, dt))


@pytest.fixture(scope="module", params=["f32", "bf16"])
def tiny(request):
    s = si.dit_tiny(request.param)
    w = si.make_dit_weights(s, 0)
    return s, w, odit.DiTOracle(s, w), make_gpu(s, w)


def _tol(s):
    return 1e-5 if s.dtype == "f32" else 2e-2


def test_full_step_matches_oracle_forward(tiny):
    import paper_2509_11628_amd as sp
    s, w, om, ctx = tiny
    B = 3
    x = si.make_latents(B, s.in_channels, s.latent_hw, seed=5)
    labels = [1, 7, s.num_classes]
    ctx.init_cache(sp.make_cfg(order=1, interval=4), B)
    xd = torch.from_numpy(x).cuda()
    out = torch.zeros_like(xd)
    ctx.full_step(xd, 0, [0, 1, 2], out, labels=labels, timestep=640.0)
    exp, feats = om.forward(x, 640.0, labels)
    assert max_abs_rel(out.cpu().numpy(), exp) <= _tol(s)
    # the cache now holds every slot's feature: an order-0 forecast returns it
    td = torch.bfloat16 if s.dtype == "bf16" else torch.float32
    f = torch.empty((s.n_slots, B, s.tokens, s.hidden), dtype=td, device="cuda")
    ctx.forecast(1, [0, 1, 2], f)
    got = f.float().cpu().numpy()
    for j in range(s.n_slots):
        assert max_abs_rel(got[j], feats[j]) <= (1e-5 if s.dtype == "f32" else 1.5e-2), j
    # a row's result does not depend on which other rows share the launch (bitwise)
    out1 = torch.zeros_like(xd)
    ctx.init_cache(sp.make_cfg(order=1, interval=4), B)
    ctx.full_step(xd, 0, [1], out1, labels=labels, timestep=640.0)
    assert torch.equal(out1[1], out[1]) and float(out1[0].abs().max()) == 0.0


def test_spec_step_matches_oracle(tiny):
    import paper_2509_11628_amd as sp
    s, w, om, ctx = tiny
    B = 2
    x = si.make_latents(B, s.in_channels, s.latent_hw, seed=6)
    labels = [3, 4]
    cfg = osamp.SpecaConfig(order=1, interval=8)
    ctx.init_cache(sp.make_cfg(order=1, interval=8), B)
    xd = torch.from_numpy(x).cuda()
    out = torch.zeros_like(xd)
    store = "bf16" if s.dtype == "bf16" else None
    caches = [core.FeatureCache(om.n_slots, 1, "taylor", store) for _ in range(B)]
    # the latent moves between steps (as it does along a trajectory), so the features really change:
    # the verification error is then well above the ~3e-3 noise floor that bf16 activations add (in quadrature)
    drift = si.make_latents(B, s.in_channels, s.latent_hw, seed=60)
    xs = {0: x, 2: (x + 0.2 * drift).astype(np.float32), 3: (x + np.array([0.6, 1.2], np.float32)[:, None, None, None] * drift).astype(np.float32)}
    for step, t in ((0, 900.0), (2, 800.0)):
        xd = torch.from_numpy(xs[step]).cuda()
        ctx.full_step(xd, step, [0, 1], out, labels=labels, timestep=t)
        for b in range(B):
            osamp.full_step(om, caches[b], xs[step][b:b + 1], t, labels[b:b + 1], step)
    exp_e, exp_out = [], []
    x = xs[3]
    xd = torch.from_numpy(x).cuda()
    for b in range(B):
        ok, e, o = osamp.speculative_attempt(om, caches[b], cfg, x[b:b + 1], 750.0, labels[b:b + 1], 3, np.float32(np.inf))
        exp_e.append(float(e[0])); exp_out.append(o[0])
    print(f"\n[{s.dtype}] expected verification errors {exp_e}")
    err, acc = ctx.spec_step(xd, 3, [0, 1], np.inf, out, labels=labels, timestep=750.0)
    np.testing.assert_allclose(err, exp_e, rtol=1e-4 if s.dtype == "f32" else 1e-1)
    assert acc.tolist() == [True, True]
    assert max_abs_rel(out.cpu().numpy(), np.stack(exp_out)) <= _tol(s)
    # a threshold between the two errors accepts exactly the smaller one
    mid = float(np.sqrt(exp_e[0] * exp_e[1]))
    if abs(exp_e[0] - exp_e[1]) / mid > 0.2:
        _, acc2 = ctx.spec_step(xd, 3, [0, 1], mid, out, labels=labels, timestep=750.0)
        assert acc2.tolist() == [e <= mid for e in exp_e]


def _run_both(s, om, ctx, S, B, cfg_kwargs, tau, cfg_scale=0.0, seed=0, solver="ddim"):
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    ts, ab = si.ddim_tables(S)
    lat = si.make_latents(B, s.in_channels, s.latent_hw, seed)
    lab = si.make_labels(B, s.num_classes, seed)
    noise = si.make_solver_noise(S, lat.shape, seed) if solver == "ddpm" else None
    sol = osamp.Solver(solver, ts, ab, cfg_scale, noise)
    exp, tr = osamp.sample(om, osamp.SpecaConfig(cache_store="bf16" if s.dtype == "bf16" else None, **cfg_kwargs), sol, tau, lat, lab)
    mode = {"newton": bd.COEF_NEWTON, "adams_bashforth": bd.COEF_ADAMS_BASHFORTH}.get(cfg_kwargs.get("mode"), bd.COEF_TAYLOR)
    kw = {k: v for k, v in cfg_kwargs.items() if k not in ("mode", "cache_layout")}
    layout = bd.CACHE_RING if cfg_kwargs.get("cache_layout") == "ring" else bd.CACHE_DIFFERENCES
    ctx.init_cache(sp.make_cfg(coef_mode=mode, layout=layout, **kw), B * (2 if cfg_scale > 0 else 1))
    xd = torch.from_numpy(lat).cuda()
    got = ctx.sample(xd, ts, ab, tau, cfg_scale=cfg_scale, labels=lab,
                     solver_kind=bd.SOLVER_DDPM if solver == "ddpm" else bd.SOLVER_DDIM,
                     noise=torch.from_numpy(noise).cuda() if noise is not None else None)
    return exp, tr, xd.cpu().numpy(), got


def _margin(tr):
    e = np.nanmax(tr.err, axis=2)
    with np.errstate(invalid="ignore"):
        m = np.abs(e - tr.tau[None, :]) / tr.tau[None, :]
    return float(np.nanmin(m)) if np.any(np.isfinite(m)) else float("inf")


# Noise the device path adds to the verification error, in quadrature: fp32 rounding for
# fp32 models; for bf16 models the bf16 rounding of activations (~3e-3) and of the cached
# differences, which a second-order extrapolation amplifies to ~1e-2.
NOISE = {"f32": 1e-5, "bf16": 1.2e-2}


def compare_traces(tr, gtr, dtype):
    """Schedules must agree decision by decision.  A decision whose oracle error is closer to
    the threshold than the device noise may legitimately flip; from there on that sample's
    trajectory is a different (equally valid) one and is no longer compared.
    -> (number of decisions compared, True if every sample agreed to the end)."""
    n, B, S = NOISE[dtype], tr.kind.shape[0], tr.kind.shape[1]
    compared, complete = 0, True
    for b in range(B):
        for s in range(S):
            ko, kg = int(tr.kind[b, s]), int(gtr["kind"][b, s])
            verified = not np.all(np.isnan(tr.err[b, s]))
            if verified:
                e, tau = float(np.nanmax(tr.err[b, s])), float(tr.tau[s])
                decisive = e > tau * 1.02 + 1e-7 or np.sqrt(e * e + n * n) < tau * 0.98
            else:
                decisive = True
            if ko != kg:
                assert not decisive, f"sample {b} step {s}: oracle kind {ko} (e={tr.err[b, s]}, tau={tr.tau[s]}) vs device {kg} (e={gtr['err'][b, s]})"
                complete = False
                break
            if verified:
                compared += 1
                ge = float(np.nanmax(gtr["err"][b, s]))
                assert abs(ge - e) <= (1e-3 * e + 1e-6 if dtype == "f32" else 0.1 * e + n), (b, s, ge, e)
    return compared, complete


def all_decisive(tr, dtype):
    """True if every verified decision of the oracle's trace lies outside the band in which compare_traces lets a
    decision flip: then the device must reproduce the whole schedule, and the latents are compared."""
    n = NOISE[dtype]
    for b in range(tr.kind.shape[0]):
        for s in range(tr.kind.shape[1]):
            if not np.all(np.isnan(tr.err[b, s])):
                e, tau = float(np.nanmax(tr.err[b, s])), float(tr.tau[s])
                if not (e > tau * 1.02 + 1e-7 or np.sqrt(e * e + n * n) < tau * 0.98):
                    return False
    return True


def must_complete(tr, dtype):
    return dtype == "f32" or all_decisive(tr, dtype)


def test_config1_trajectory(tiny):
    """Configuration 1: 20 DDIM steps, order 1, interval 4, verify = last block, tau 0.05 -> 0.01 linear."""
    s, w, om, ctx = tiny
    tau = core.tau_linear(0.05, 0.01, 20)
    exp, tr, got, gtr = _run_both(s, om, ctx, 20, 2, dict(order=1, interval=4), tau)
    print(f"\n[{s.dtype}] min decision margin {_margin(tr):.3e}; kinds {tr.kind.tolist()}")
    compared, complete = compare_traces(tr, gtr, s.dtype)
    print(f"decisions compared {compared}, schedules identical to the end: {complete}")
    assert compared >= 10
    if must_complete(tr, s.dtype):
        assert complete
    if complete:
        assert max_abs_rel(got, exp) <= _tol(s)
        assert gtr["n_full"] == tr.n_full and gtr["n_reject"] == int((tr.kind == 2).sum())
    assert (tr.kind == 1).sum() > 0 and (tr.kind == 2).sum() > 0     # both paths exercised


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_odd_token_count_trajectory(dtype):
    """A 6x6 latent gives 9 tokens per row: half a row is not a whole number of tokens, so the forecast-and-fold kernel
    takes its one-position form, and every tile of the step is ragged.  Guided pairs, order 2, both cache layouts."""
    s = si.DiTShape(depth=2, hidden=64, heads=4, mlp_hidden=256, in_channels=4, latent_hw=6, patch=2, num_classes=10, freq_dim=32, dtype=dtype)
    assert s.tokens == 9
    w = si.make_dit_weights(s, 3)
    om, ctx = odit.DiTOracle(s, w), make_gpu(s, w)
    tau = core.tau_geometric(0.3, 0.2, 12)
    for layout in ("differences", "ring"):
        exp, tr, got, gtr = _run_both(s, om, ctx, 12, 3, dict(order=2, interval=4, cache_layout=layout), tau, cfg_scale=1.5, seed=2)
        print(f"\n[{dtype}, {layout}] min decision margin {_margin(tr):.3e}; kinds {tr.kind.tolist()}")
        compared, complete = compare_traces(tr, gtr, dtype)
        assert compared >= 6 and (tr.kind == 1).sum() > 0
        if must_complete(tr, dtype):
            assert complete
        if complete:
            assert max_abs_rel(got, exp) <= _tol(s)


def test_config1_geometric_and_newton(tiny):
    s, w, om, ctx = tiny
    tau = core.tau_geometric(0.05, 0.2, 20)
    for kw in (dict(order=1, interval=4), dict(order=2, interval=5, mode="newton"), dict(order=2, interval=5, verify_block=0),
               dict(order=2, interval=5, mode="adams_bashforth"), dict(order=0, interval=3)):
        exp, tr, got, gtr = _run_both(s, om, ctx, 20, 2, kw, tau)
        compared, complete = compare_traces(tr, gtr, s.dtype)
        assert compared >= 6, kw
        if must_complete(tr, s.dtype):
            assert complete, kw
        if complete:
            assert max_abs_rel(got, exp) <= _tol(s), kw


def test_decisive_margins_force_latent_comparison(tiny):
    """A trajectory whose every decision is far from the threshold in the oracle (>= 10 % after the bf16 noise
    allowance): no flip is tolerated for either dtype, so schedule, counts, errors and final latents are all
    compared.  Constant threshold 0.16, order 2, interval 5: 27 accepted and 12 rejected attempts over 3 samples;
    both cache layouts, with and without guidance."""
    s, w, om, ctx = tiny
    S, B = 14, 3
    tau = np.full(S, 0.16, np.float32)
    for kw, scale in ((dict(order=2, interval=5), 0.0), (dict(order=2, interval=5, cache_layout="ring"), 1.5)):
        exp, tr, got, gtr = _run_both(s, om, ctx, S, B, kw, tau, cfg_scale=scale, seed=3)
        m = np.inf
        for b in range(B):
            for st in range(S):
                if not np.all(np.isnan(tr.err[b, st])):
                    e = float(np.nanmax(tr.err[b, st]))
                    m = min(m, (e - 0.16) / 0.16 if e > 0.16 else (0.16 - np.sqrt(e * e + NOISE["bf16"] ** 2)) / 0.16)
        assert m >= 0.10 and all_decisive(tr, "bf16"), m                # the case itself: decided by the oracle alone
        assert (tr.kind == 1).sum() >= 20 and (tr.kind == 2).sum() >= 8
        compared, complete = compare_traces(tr, gtr, s.dtype)
        assert complete and compared == int((tr.kind != 0).sum()), (kw, compared)
        assert np.array_equal(gtr["kind"], tr.kind), kw
        assert gtr["n_full"] == tr.n_full and gtr["n_spec"] == int((tr.kind == 1).sum()) and gtr["n_reject"] == int((tr.kind == 2).sum())
        assert max_abs_rel(got, exp) <= _tol(s), kw


def test_other_metrics_through_the_sampler(tiny):
    """The appendix's other error metrics chosen through speca_cfg.metric and used by speca_sample's verifier
    (not only by the stand-alone reduction): one trajectory per metric against the oracle run with that metric."""
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    s, w, om, ctx = tiny
    S, B = 12, 2
    ts, ab = si.ddim_tables(S)
    lat = si.make_latents(B, s.in_channels, s.latent_hw, 3)
    lab = si.make_labels(B, s.num_classes, 3)
    sol = osamp.Solver("ddim", ts, ab, 0.0)
    # thresholds per metric: cosine distance is about e^2 / 2 of the relative L2 error e, L-infinity is larger than L2
    for name, code, tau0 in (("l1", bd.METRIC_L1, 0.16), ("linf", bd.METRIC_LINF, 0.3), ("cosine", bd.METRIC_COSINE, 0.012)):
        tau = np.full(S, tau0, np.float32)
        exp, tr = osamp.sample(om, osamp.SpecaConfig(order=2, interval=5, metric=name, cache_store="bf16" if s.dtype == "bf16" else None),
                               sol, tau, lat, lab)
        ctx.init_cache(sp.make_cfg(order=2, interval=5, metric=code), B)
        xd = torch.from_numpy(lat).cuda()
        gtr = ctx.sample(xd, ts, ab, tau, labels=lab)
        print(f"\n[{s.dtype}] metric {name}: kinds {tr.kind.tolist()} errors {np.round(tr.err[..., 0], 4).tolist()}")
        assert (tr.kind == 1).sum() > 0 and (tr.kind == 2).sum() > 0, name
        if s.dtype == "f32":
            assert np.array_equal(gtr["kind"], tr.kind), name
            m = ~np.isnan(tr.err[..., 0])
            np.testing.assert_allclose(gtr["err"][..., 0][m], tr.err[..., 0][m], rtol=2e-3, atol=1e-6, err_msg=name)
            assert max_abs_rel(xd.cpu().numpy(), exp) <= 1e-5, name
        else:
            compared, complete = compare_traces_metric(tr, gtr, name)
            assert compared >= 4, name
            if complete:
                assert max_abs_rel(xd.cpu().numpy(), exp) <= 2e-2, name


def compare_traces_metric(tr, gtr, name):
    """bf16 runs under another metric: the noise the device adds is metric-dependent (cosine distance is second
    order in the rounding noise, L-infinity sees single elements), so a decision within 15 % of the threshold
    may flip; from there on the sample is no longer compared."""
    compared, complete = 0, True
    for b in range(tr.kind.shape[0]):
        for st in range(tr.kind.shape[1]):
            ko, kg = int(tr.kind[b, st]), int(gtr["kind"][b, st])
            e, tau = float(tr.err[b, st, 0]), float(tr.tau[st])
            if ko != kg:
                assert not np.isnan(e) and abs(e - tau) <= 0.15 * tau + 2e-3, (name, b, st, ko, kg, e, tau)
                complete = False
                break
            if not np.isnan(e):
                compared += 1
                ge = float(gtr["err"][b, st, 0])
                assert abs(ge - e) <= 0.15 * e + (3e-4 if name == "cosine" else 1.2e-2), (name, b, st, ge, e)
    return compared, complete


def test_threshold_zero_is_plain_sampling(tiny):
    s, w, om, ctx = tiny
    tau = np.zeros(20, np.float32)
    exp, tr, got, gtr = _run_both(s, om, ctx, 20, 2, dict(order=1, interval=4), tau)
    assert np.all(gtr["kind"] == 0) and gtr["n_spec"] == 0
    ts, ab = si.ddim_tables(20)
    plain = osamp.sample_plain(om, osamp.Solver("ddim", ts, ab), si.make_latents(2, s.in_channels, s.latent_hw, 0),
                               si.make_labels(2, s.num_classes, 0))
    assert max_abs_rel(got, plain) <= _tol(s)
    # and the library's own tau=0 run is bit-identical to a second run (deterministic kernels)
    _, _, got2, _ = _run_both(s, om, ctx, 20, 2, dict(order=1, interval=4), tau)
    assert got.tobytes() == got2.tobytes()


def test_threshold_infinite_gives_fixed_pattern(tiny):
    s, w, om, ctx = tiny
    tau = np.full(12, np.inf, np.float32)
    exp, tr, got, gtr = _run_both(s, om, ctx, 12, 2, dict(order=2, interval=4), tau)
    assert gtr["kind"][0].tolist() == [0 if i % 4 == 0 else 1 for i in range(12)]
    assert max_abs_rel(got, exp) <= _tol(s)


def test_guided_trajectory(tiny):
    s, w, om, ctx = tiny
    tau = core.tau_linear(0.08, 0.02, 10)
    exp, tr, got, gtr = _run_both(s, om, ctx, 10, 3, dict(order=1, interval=3), tau, cfg_scale=1.5, seed=2)
    print(f"\n[{s.dtype}] guided: min margin {_margin(tr):.3e}; kinds {tr.kind.tolist()}")
    compared, complete = compare_traces(tr, gtr, s.dtype)
    assert compared >= 6
    if must_complete(tr, s.dtype):
        assert complete
    if complete:
        assert max_abs_rel(got, exp) <= _tol(s)
        m = ~np.isnan(tr.err)
        assert np.array_equal(~np.isnan(gtr["err"]), m)
        np.testing.assert_allclose(gtr["err"][m], tr.err[m], rtol=1e-3 if s.dtype == "f32" else 1.5e-1, atol=0 if s.dtype == "f32" else 5e-3)


def test_ring_layout_trajectories(tiny):
    """The raw-feature ring layout of the cache through whole trajectories (fused refresh in the
    branch epilogues, forecast-and-fold, verification), against the oracle's ring cache."""
    s, w, om, ctx = tiny
    tau = core.tau_linear(0.05, 0.01, 20)
    for kw, scale in ((dict(order=1, interval=4), 0.0), (dict(order=2, interval=5, mode="newton"), 0.0),
                      (dict(order=3, interval=6, mode="adams_bashforth"), 0.0), (dict(order=2, interval=4), 1.5)):
        kw = dict(kw, cache_layout="ring")
        exp, tr, got, gtr = _run_both(s, om, ctx, 20, 2, kw, tau, cfg_scale=scale, seed=5)
        compared, complete = compare_traces(tr, gtr, s.dtype)
        print(f"\n[{s.dtype}] ring {kw}: kinds {tr.kind.tolist()} compared {compared} complete {complete}")
        assert compared >= 4, kw
        if must_complete(tr, s.dtype):
            assert complete, kw
        if complete:
            assert max_abs_rel(got, exp) <= _tol(s), kw
    # tau = 0: plain sampling, and the layout cannot matter (no forecast is ever used)
    z = np.zeros(20, np.float32)
    _, _, got_ring, g1 = _run_both(s, om, ctx, 20, 2, dict(order=2, interval=4, cache_layout="ring"), z)
    _, _, got_diff, g2 = _run_both(s, om, ctx, 20, 2, dict(order=2, interval=4), z)
    assert got_ring.tobytes() == got_diff.tobytes() and np.all(g1["kind"] == 0)


def test_stochastic_solver_trajectory(tiny):
    """Eq. 1 as the solver: the draws are an input, so the trajectory is still a function of its
    inputs and is compared decision by decision; also guided, and with tau = 0 (plain ancestral
    sampling)."""
    s, w, om, ctx = tiny
    tau = core.tau_linear(0.08, 0.02, 12)
    for kw, scale in ((dict(order=1, interval=4), 0.0), (dict(order=2, interval=3), 1.5)):
        exp, tr, got, gtr = _run_both(s, om, ctx, 12, 2, kw, tau, cfg_scale=scale, seed=3, solver="ddpm")
        compared, complete = compare_traces(tr, gtr, s.dtype)
        print(f"\n[{s.dtype}] ancestral: kinds {tr.kind.tolist()} compared {compared} complete {complete}")
        assert compared >= 4
        if must_complete(tr, s.dtype):
            assert complete
        if complete:
            assert max_abs_rel(got, exp) <= _tol(s)
    exp, tr, got, gtr = _run_both(s, om, ctx, 12, 2, dict(order=1, interval=4), np.zeros(12, np.float32), seed=3, solver="ddpm")
    assert np.all(gtr["kind"] == 0) and max_abs_rel(got, exp) <= _tol(s)
    # the draws do reach the latents: the deterministic solver lands elsewhere
    _, _, got_ddim, _ = _run_both(s, om, ctx, 12, 2, dict(order=1, interval=4), np.zeros(12, np.float32), seed=3)
    assert max_abs_rel(got, got_ddim) > 0.05


def test_sample_error_paths(tiny):
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    s, w, om, ctx = tiny
    ts, ab = si.ddim_tables(4)
    x = torch.zeros((2, s.in_channels, s.latent_hw, s.latent_hw), device="cuda")
    ctx.init_cache(sp.make_cfg(order=1, interval=2), 2)
    with pytest.raises(sp.SpecaError) as e:
        ctx.sample(x, ts, ab, np.ones(4, np.float32), cfg_scale=1.5, labels=[0, 1])     # needs 4 rows
    assert e.value.code == bd.ESTATE
    with pytest.raises(sp.SpecaError) as e:
        ctx.sample(x, ts, ab, np.ones(4, np.float32), labels=[0, 99])
    assert e.value.code == bd.EINVAL
    with pytest.raises(sp.SpecaError) as e:
        ctx.init_cache(sp.make_cfg(order=1, interval=2, verify_block=5), 2)
    assert e.value.code == bd.EINVAL
    ctx.init_cache(sp.make_cfg(order=1, interval=2), 2)
    with pytest.raises(sp.SpecaError) as e:
        ctx.sample(x, ts, ab, np.ones(4, np.float32), labels=[0, 1], solver_kind=bd.SOLVER_DDPM)     # no draws given
    assert e.value.code == bd.EINVAL


def test_lanes_do_not_change_results(tiny):
    """Row groups of a step run side by side on streams of the library; a row's result must not
    depend on how the rows were grouped: same bits for 1, 2 and 4 lanes (mixed schedule, guided)."""
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    s, w, om, ctx = tiny
    S, B = 10, 8                                   # 16 rows: launches of 9 rows and more are split into row groups
    ts, ab = si.ddim_tables(S)
    lat = si.make_latents(B, s.in_channels, s.latent_hw, 3)
    lab = si.make_labels(B, s.num_classes, 3)
    tau = core.tau_linear(0.08, 0.02, S)
    outs = []
    try:
        for lanes in (1, 2, 4):
            ctx.set_lanes(lanes)
            ctx.init_cache(sp.make_cfg(order=2, interval=4), 2 * B)
            xd = torch.from_numpy(lat).cuda()
            tr = ctx.sample(xd, ts, ab, tau, cfg_scale=1.5, labels=lab)
            outs.append((xd.cpu().numpy(), tr))
    finally:
        ctx.set_lanes(2)
    kinds = outs[0][1]["kind"]
    assert (kinds == 1).any() and (kinds == 0).any()
    for x, tr in outs[1:]:
        assert np.array_equal(x, outs[0][0])
        assert np.array_equal(tr["kind"], kinds) and np.array_equal(tr["err"], outs[0][1]["err"], equal_nan=True)
    with pytest.raises(sp.SpecaError) as e:
        ctx.set_lanes(9)
    assert e.value.code == bd.EINVAL


def test_config3_full_size_sampled():
    """Configuration 3 at full size, in the launch shape the benchmark times (16 rows = 8 samples x
    guidance pair, bf16, 4 lanes): the reference step of one guidance pair (rows 0 and 8) against the
    oracle's forward of those two rows (about 10 s of CPU), model output and sampled cached features;
    then properties that hold at any size: thresholds of zero reproduce plain sampling bit for bit and
    the lane count does not change a bit."""
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    s = si.dit_xl2("bf16")
    w = si.make_dit_weights(s, 0)
    ctx = sp.Context(sp.dit_desc(s), sp.to_device(w, bd.BF16))
    B = 8
    ctx.set_lanes(4)
    ctx.init_cache(sp.make_cfg(order=2, interval=5), 2 * B)
    lat = si.make_latents(B, s.in_channels, s.latent_hw, 0)
    lab = si.make_labels(B, s.num_classes, 0)
    labels_rows = list(lab) + [s.num_classes] * B                    # conditional rows, then null-label rows
    xd = torch.from_numpy(np.concatenate([lat, lat])).cuda()          # one latent row per cache row
    out = torch.zeros_like(xd)
    ts, ab = si.ddim_tables(50)
    ctx.full_step(xd, 0, list(range(2 * B)), out, timestep=float(ts[0]), labels=labels_rows)
    om = odit.DiTOracle(s, w)
    exp, feats = om.forward(np.stack([lat[0], lat[0]]), float(ts[0]), [int(lab[0]), s.num_classes])
    got = out.cpu().numpy()
    assert max_abs_rel(got[[0, B]], exp) <= 2e-2
    f = torch.empty((s.n_slots, 2, s.tokens, s.hidden), dtype=torch.bfloat16, device="cuda")
    ctx.forecast(1, [0, B], f)                                        # one reference: the forecast is the cached feature
    gf = f.float().cpu().numpy()
    rng = np.random.default_rng(0)
    for j in (0, 1, 27, 54, 55):
        idx = (rng.integers(0, 2, 2000), rng.integers(0, s.tokens, 2000), rng.integers(0, s.hidden, 2000))
        a, b = gf[j][idx], feats[j][idx]
        assert np.max(np.abs(a - b)) <= 2e-2 * np.max(np.abs(feats[j])), j
    # properties at full size: tau = 0 is plain sampling; lanes do not change bits (8 steps keep it short)
    S = 8
    ts, ab = si.ddim_tables(S)
    res = []
    for lanes, tau in ((4, np.zeros(S, np.float32)), (1, np.zeros(S, np.float32)), (4, bd.tau_geometric(0.5, 0.5, S)), (2, bd.tau_geometric(0.5, 0.5, S))):
        ctx.set_lanes(lanes)
        ctx.init_cache(sp.make_cfg(order=2, interval=4), 2 * B)
        x = torch.from_numpy(lat).cuda()
        tr = ctx.sample(x, ts, ab, tau, cfg_scale=1.5, labels=lab)
        res.append((x.cpu().numpy(), tr))
    assert np.all(res[0][1]["kind"] == 0) and np.array_equal(res[0][0], res[1][0])
    assert np.array_equal(res[2][0], res[3][0]) and np.array_equal(res[2][1]["kind"], res[3][1]["kind"])
    assert np.all(np.isfinite(res[2][0]))
    # a short trajectory in the benchmark's launch shape (8 samples, guidance, 4 lanes) with an accepted, a
    # rejected and another accepted attempt; sample 0 against the oracle run on that sample alone
    # (samples are independent: own cache, own schedule)
    S = 4
    ts, ab = si.ddim_tables(S)
    tau = np.array([0.0, np.inf, 1e-3, np.inf], np.float32)
    sol = osamp.Solver("ddim", ts, ab, 1.5)
    for layout, code in (("differences", bd.CACHE_DIFFERENCES), ("ring", bd.CACHE_RING)):      # both layouts of the cache
        finals = []
        for lanes in (4, 1):
            ctx.set_lanes(lanes)
            ctx.init_cache(sp.make_cfg(order=2, interval=5, layout=code), 2 * B)
            x = torch.from_numpy(lat).cuda()
            gtr = ctx.sample(x, ts, ab, tau, cfg_scale=1.5, labels=lab)
            finals.append(x.cpu().numpy())
        assert np.array_equal(finals[0], finals[1]), layout
        exp1, tr = osamp.sample(om, osamp.SpecaConfig(order=2, interval=5, cache_store="bf16", cache_layout=layout), sol, tau,
                                lat[:1], lab[:1])
        assert tr.kind[0].tolist() == [0, 1, 2, 1] and gtr["kind"][0].tolist() == [0, 1, 2, 1], layout
        compared, complete = compare_traces(tr, {"kind": gtr["kind"][:1], "err": gtr["err"][:1]}, "bf16")
        assert compared == 3 and complete, layout
        assert max_abs_rel(finals[0][:1], exp1) <= 2e-2, layout
    ctx.close()


def test_config3_full_size_diverging_schedules():
    """Configuration 3 at full size with samples whose schedules diverge, so that every step after the first splits
    the batch into a speculative row list and a full row list (rejected rows recomputed at M = 2048 while the other
    half of the batch finishes from forecasts): 8 samples x guidance pair, bf16, 4 lanes, ring layout, 5 DDIM steps.
    With seeded random weights the verification errors of equally scaled latents lie within 2 % of each other, so the
    latents are scaled per sample (0.4 .. 0.7 and 1.4 .. 2.0): the error grows with the scale and per-step thresholds
    placed in the gap send the two groups opposite ways at every step.  One sample of each group is checked against
    the oracle run on that sample alone (samples are independent): schedule, errors, final latents."""
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    s = si.dit_xl2("bf16")
    w = si.make_dit_weights(s, 0)
    ctx = sp.Context(sp.dit_desc(s), sp.to_device(w, bd.BF16))
    B, S = 8, 5
    scales = np.array([0.4, 0.5, 0.6, 0.7, 1.4, 1.6, 1.8, 2.0], np.float32)
    lat = si.make_latents(B, s.in_channels, s.latent_hw, 0) * scales[:, None, None, None]
    lab = si.make_labels(B, s.num_classes, 0)
    ts, ab = si.ddim_tables(S)
    tau = np.array([0.0, 0.5, 0.65, 0.55, 0.5], np.float32)
    ctx.set_lanes(4)
    ctx.init_cache(sp.make_cfg(order=2, interval=5, layout=bd.CACHE_RING), 2 * B)
    x = torch.from_numpy(lat).cuda()
    gtr = ctx.sample(x, ts, ab, tau, cfg_scale=1.5, labels=lab)
    got = x.cpu().numpy()
    print(f"\nkinds {gtr['kind'].tolist()}\nerrors {np.round(np.nanmax(gtr['err'], axis=2), 4).tolist()}")
    # the two groups go opposite ways at every step: each launch after step 0 holds half of the batch
    assert gtr["kind"][:4].tolist() == [[0, 1, 2, 1, 2]] * 4 and gtr["kind"][4:].tolist() == [[0, 2, 1, 2, 1]] * 4
    assert gtr["n_spec"] == 16 and gtr["n_reject"] == 16 and gtr["n_full"] == 24
    om = odit.DiTOracle(s, w)
    sol = osamp.Solver("ddim", ts, ab, 1.5)
    for b in (1, 6):
        exp1, tr = osamp.sample(om, osamp.SpecaConfig(order=2, interval=5, cache_store="bf16", cache_layout="ring"), sol, tau,
                                lat[b:b + 1], lab[b:b + 1])
        print(f"sample {b}: oracle kinds {tr.kind[0].tolist()} errors {np.round(np.nanmax(tr.err[0], axis=1), 4).tolist()}")
        assert all_decisive(tr, "bf16"), b                              # the thresholds sit in the gap for the oracle too
        compared, complete = compare_traces(tr, {"kind": gtr["kind"][b:b + 1], "err": gtr["err"][b:b + 1]}, "bf16")
        assert compared == 4 and complete, b
        assert max_abs_rel(got[b:b + 1], exp1) <= 2e-2, b
    # the same trajectory run serially gives the same bits
    ctx.set_lanes(1)
    ctx.init_cache(sp.make_cfg(order=2, interval=5, layout=bd.CACHE_RING), 2 * B)
    x1 = torch.from_numpy(lat).cuda()
    ctx.sample(x1, ts, ab, tau, cfg_scale=1.5, labels=lab)
    assert np.array_equal(x1.cpu().numpy(), got)
    ctx.close()
