"""Pins of the oracle's forecast / difference / verification arithmetic against
what the paper and the mathematics fix (no GPU, no library)."""
import math

import numpy as np
import pytest

from oracle import speca_core as core


def _cache_from(fn, steps, m, mode, store=None):
    c = core.FeatureCache(1, m, mode, store)
    for s in steps:
        c.refresh(s, [np.asarray(fn(s), dtype=np.float64)])
    return c


# --- worked examples, by hand (Sec. 3.3, Eq. 2-3) -----------------------------------


@pytest.mark.parametrize("mode", ["taylor", "newton"])
def test_linear_worked_example(mode):
    # F(u) = 3u+1, full steps at u=0 and u=4 (N=4): F=1, 13; first difference 12.
    # Forecast two steps ahead: 13 + (2/4)*12 = 19 = F(6).
    c = _cache_from(lambda u: np.array([3.0 * u + 1.0]), [0, 4], 1, mode)
    assert c.forecast(6, 0)[0] == pytest.approx(19.0, abs=1e-12)
    # stored difference is the slope per step
    assert c.D[0][1][0] == pytest.approx(3.0, abs=1e-12)


def test_quadratic_worked_example_golden():
    # tests/golden/quadratic_example.txt: F(u)=u^2 at u=0,4,8 -> F=0,16,64,
    # backward differences 48 and 32.  Eq. 2 as printed gives 64+12+1=77 at k=1
    # and 64+36+9=109 at k=3; the exact values are 81 and 121 (deficit c*k*N).
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "quadratic_example.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                mode, k, val = line.split()
                rows[(mode, int(k))] = float(val)
    for (mode, k), val in rows.items():
        c = _cache_from(lambda u: np.array([float(u * u)]), [0, 4, 8], 2, mode)
        assert c.forecast(8 + k, 0)[0] == pytest.approx(val, abs=1e-10), (mode, k)


def test_eq2_literal_signs():
    # Eq. 2-3 evaluated literally in the paper's indexing (timestep decreasing):
    # features latest first = F(x_t), F(x_{t+N}), F(x_{t+2N}) = 64, 16, 0.
    feats = [np.array([64.0]), np.array([16.0]), np.array([0.0])]
    assert core.finite_difference_eq3(feats, 1)[0] == -48.0      # (-1)^(1-0) F_t + F_{t+N}
    assert core.finite_difference_eq3(feats, 2)[0] == 32.0
    assert core.taylor_forecast_eq2(feats, N=4, k=1, m=2)[0] == pytest.approx(77.0)
    assert core.taylor_forecast_eq2(feats, N=4, k=3, m=2)[0] == pytest.approx(109.0)
    assert core.taylor_forecast_eq2(feats, N=4, k=2, m=1)[0] == pytest.approx(64 + 24.0)


# --- polynomial exactness -------------------------------------------------------------


@pytest.mark.parametrize("m", [0, 1, 2, 3])
def test_newton_exact_on_polynomials_irregular_gaps(m):
    rng = np.random.default_rng(m)
    coef = rng.standard_normal((m + 1, 7))
    fn = lambda u: sum(coef[d] * float(u) ** d for d in range(m + 1))
    steps = [0, 3, 4, 9, 11][: m + 1]
    c = _cache_from(fn, steps, m, "newton")
    for k in (1, 2, 5):
        s = steps[-1] + k
        np.testing.assert_allclose(c.forecast(s, 0), fn(s), rtol=1e-10, atol=1e-10)


@pytest.mark.parametrize("m", [1, 2, 3])
def test_taylor_exact_up_to_degree_one(m):
    rng = np.random.default_rng(10 + m)
    a, b = rng.standard_normal(5), rng.standard_normal(5)
    fn = lambda u: a + b * u
    c = _cache_from(fn, [0, 2, 7, 9][: m + 1], m, "taylor")       # irregular gaps
    s = c.refs[0] + 3
    np.testing.assert_allclose(c.forecast(s, 0), fn(s), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("N,k", [(4, 1), (4, 3), (5, 2), (3, 2)])
def test_taylor_quadratic_deficit_is_ckN(N, k):
    # one-sided slope instead of the derivative: the printed formula misses a
    # quadratic a+bu+cu^2 by exactly c*k*N on a uniform grid
    rng = np.random.default_rng(N * 10 + k)
    a, b, cc = rng.standard_normal(4), rng.standard_normal(4), rng.standard_normal(4)
    fn = lambda u: a + b * u + cc * u * u
    steps = [2, 2 + N, 2 + 2 * N]
    c = _cache_from(fn, steps, 2, "taylor")
    s = steps[-1] + k
    np.testing.assert_allclose(fn(s) - c.forecast(s, 0), cc * k * N, rtol=1e-9, atol=1e-9)


def test_modes_identical_up_to_order_one():
    rng = np.random.default_rng(3)
    f = [rng.standard_normal(6) for _ in range(2)]
    for m in (0, 1):
        ct = core.FeatureCache(1, m, "taylor"); cn = core.FeatureCache(1, m, "newton")
        for s, x in zip([0, 3], f):
            ct.refresh(s, [x]); cn.refresh(s, [x])
        np.testing.assert_allclose(ct.forecast(5, 0), cn.forecast(5, 0), rtol=1e-13)


# --- recursion vs Eq. 3 written out -----------------------------------------------------


@pytest.mark.parametrize("m,N", [(1, 4), (2, 4), (3, 2), (2, 5)])
def test_recursion_reduces_to_eq3_on_uniform_grid(m, N):
    rng = np.random.default_rng(m * 7 + N)
    raw = [rng.standard_normal((3, 5)) for _ in range(m + 3)]       # more refs than kept
    c = core.FeatureCache(1, m, "taylor")
    for j, f in enumerate(raw):
        c.refresh(j * N, [f])
    latest_first = raw[::-1]
    for i in range(m + 1):
        # stored D^i * N^i  ==  (-1)^i * Eq.3 sum (Eq. 3 weights the latest feature (-1)^i)
        np.testing.assert_allclose(c.D[0][i] * N ** i, (-1) ** i * core.finite_difference_eq3(latest_first, i),
                                   rtol=1e-11, atol=1e-11)
    for k in range(1, N):
        np.testing.assert_allclose(c.forecast(c.refs[0] + k, 0),
                                   core.taylor_forecast_eq2(latest_first, N, k, m), rtol=1e-11, atol=1e-11)


def test_warmup_uses_available_order():
    c = core.FeatureCache(1, 2, "taylor")
    c.refresh(0, [np.array([5.0])])
    assert c.order_available == 0 and c.forecast(2, 0)[0] == 5.0            # plain reuse
    c.refresh(3, [np.array([8.0])])
    assert c.order_available == 1 and c.forecast(5, 0)[0] == pytest.approx(10.0)
    c.refresh(4, [np.array([20.0])])
    assert c.order_available == 2
    assert c.refs == [4, 3, 0]


def test_refs_keep_m_plus_one():
    c = core.FeatureCache(2, 1, "newton")
    for s in range(5):
        c.refresh(s, [np.zeros(2), np.ones(2)])
    assert c.refs == [4, 3]


# --- coefficients -----------------------------------------------------------------------


def test_coefficient_tables():
    assert core.forecast_coefficients("taylor", 11, [8, 4, 0], 2) == [1.0, 3.0, 4.5]
    assert core.forecast_coefficients("newton", 11, [8, 4, 0], 2) == [1.0, 3.0, 21.0]
    assert core.refresh_divisors("taylor", 9, [7, 4, 0], 2) == [2.0, 2.0]
    assert core.refresh_divisors("newton", 9, [7, 4, 0], 2) == [2.0, 5.0]


# --- Eq. 4 ------------------------------------------------------------------------------


def test_relative_error_hand_values():
    t = np.array([3.0, 4.0])
    assert core.relative_error(t, t) == 0.0
    assert core.relative_error(np.zeros(2), t) == pytest.approx(5.0 / (5.0 + 1e-8), rel=1e-15)
    assert core.relative_error(np.array([3.0, 4.0 + 0.5]), t) == pytest.approx(0.1, rel=1e-8)
    # zero truth: eps keeps it finite
    assert core.relative_error(np.array([1e-9, 0.0]), np.zeros(2)) == pytest.approx(0.1, rel=1e-12)


def test_relative_error_scale_invariant_and_asymmetric():
    rng = np.random.default_rng(0)
    p, t = rng.standard_normal(1000), rng.standard_normal(1000)
    e = core.relative_error(p, t)
    assert core.relative_error(7.5 * p, 7.5 * t) == pytest.approx(e, rel=1e-9)
    assert e == pytest.approx(np.linalg.norm(p - t) / np.linalg.norm(t), rel=1e-9)
    assert core.relative_error(t, p) != pytest.approx(e, rel=1e-3)         # denominator is the truth
    assert float(core.relative_error_f32(p, t)) == pytest.approx(e, rel=1e-6)


def test_other_metrics_hand_values():
    p, t = np.array([1.0, -2.0, 2.0]), np.array([1.0, -1.0, 4.0])
    assert core.relative_error_l1(p, t) == pytest.approx(3.0 / 6.0, rel=1e-8)
    assert core.relative_error_linf(p, t) == pytest.approx(2.0 / 4.0, rel=1e-8)
    assert core.cosine_distance(t, 3 * t) == pytest.approx(0.0, abs=1e-9)
    assert core.cosine_distance(np.array([1.0, 0]), np.array([0, 1.0])) == pytest.approx(1.0)


# --- sequential validation, thresholds, speed-up model -------------------------------------


def test_sequential_validation_sets():
    tau = [0.1] * 5
    assert core.sequential_validation([0.01, 0.1, 0.05, 0.02, 0.0], tau) == ([1, 2, 3, 4, 5], [])
    # first violation rejects itself and everything after, even if later errors are small
    assert core.sequential_validation([0.01, 0.02, 0.11, 0.0, 0.0], tau) == ([1, 2], [3, 4, 5])
    assert core.sequential_validation([0.2, 0.0], tau[:2]) == ([], [1, 2])
    assert core.accept(0.1, 0.1) and not core.accept(np.nextafter(np.float32(0.1), np.float32(1)), 0.1)


def test_threshold_schedules():
    tau = core.tau_geometric(0.5, 0.05, 50)
    assert tau.dtype == np.float32 and tau[0] == np.float32(0.5)
    assert tau[25] == pytest.approx(0.5 * math.sqrt(0.05), rel=1e-6)
    assert np.all(np.diff(tau) < 0)
    assert 0.5 * 0.05 < tau[-1] < 0.5 * 0.05 * 1.1                    # approaches tau0*beta, never reaches it
    lin = core.tau_linear(0.05, 0.01, 20)
    assert lin[0] == np.float32(0.05) and lin[-1] == np.float32(0.01)
    assert lin[10] == pytest.approx(0.05 - 0.04 * 10 / 19, rel=1e-6)


def test_speedup_model_matches_paper_example():
    # appendix: alpha = 0.85, gamma = 0.05 -> 1/0.1925 ~ 5.2x; alpha -> 1 gives 1/gamma
    assert core.speedup_model(0.85, 0.05) == pytest.approx(1 / 0.1925, rel=1e-12)
    assert round(core.speedup_model(0.85, 0.05), 1) == 5.2
    assert core.speedup_model(1.0, 0.05) == pytest.approx(20.0)
    assert core.speedup_model(0.5, 0.0, 0.1) == pytest.approx(1 / (1 - 0.5 * 0.9))


# --- storage rounding ---------------------------------------------------------------------


def test_bf16_round_known_values():
    r = core.bf16_round(np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -7, -3.1415926, 0.0]))
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1 + 2.0 ** -6 and r[3] == 1 + 2.0 ** -7
    assert r[4] == -3.140625 and r[5] == 0.0
    x = np.random.default_rng(0).standard_normal(1000)
    assert np.max(np.abs(core.bf16_round(x) - x) / np.abs(x)) <= 2.0 ** -8


def test_bf16_cache_close_to_exact():
    rng = np.random.default_rng(5)
    feats = [core.bf16_round(rng.standard_normal(256) + 0.1 * s) for s in (0, 4, 8)]
    ce = core.FeatureCache(1, 2, "taylor"); cb = core.FeatureCache(1, 2, "taylor", "bf16")
    for s, f in zip((0, 4, 8), feats):
        ce.refresh(s, [f]); cb.refresh(s, [f])
    np.testing.assert_array_equal(cb.D[0][0], ce.D[0][0])
    assert np.max(np.abs(cb.forecast(10, 0) - ce.forecast(10, 0))) < 2e-2


# ---- Adams-Bashforth draft policy (appendix ablation of draft models; textbook coefficients) -----------------

AB_ORDINATE_WEIGHTS = {   # y_{n+1} = y_n + h sum_j b_j f_{n-j}, classical tables
    1: [1.0],
    2: [3 / 2, -1 / 2],
    3: [23 / 12, -16 / 12, 5 / 12],
    4: [55 / 24, -59 / 24, 37 / 24, -9 / 24],
}


def test_adams_bashforth_gammas_are_the_classical_ones():
    np.testing.assert_allclose(core.adams_bashforth_gammas(5), [1, 1 / 2, 5 / 12, 3 / 8, 251 / 720], rtol=1e-14)


@pytest.mark.parametrize("q", [1, 2, 3, 4])
@pytest.mark.parametrize("g,k", [(4, 4), (3, 1), (5, 2)])
def test_adams_bashforth_equals_ordinate_form(q, g, k):
    """The forecast from the cached differences equals the method written with its classical
    weights on the raw slopes between references (uniform gaps g, one step of size k)."""
    rng = np.random.default_rng(q * 10 + g)
    steps = [g * i for i in range(q + 1)]                  # q+1 references -> q slopes
    feats = [rng.standard_normal(7) for _ in steps]
    cache = core.FeatureCache(1, q, "adams_bashforth")
    for s_, f in zip(steps, feats):
        cache.refresh(s_, [f])
    got = cache.forecast(steps[-1] + k, 0)
    latest_first = feats[::-1]
    slopes = [(latest_first[j] - latest_first[j + 1]) / g for j in range(q)]
    exp = latest_first[0] + k * sum(b * s_ for b, s_ in zip(AB_ORDINATE_WEIGHTS[q], slopes))
    np.testing.assert_allclose(got, exp, rtol=1e-12, atol=1e-12)


def test_adams_bashforth_exact_on_lines_and_differs_from_taylor_on_curves():
    a, b = 0.7, -0.3
    cache = core.FeatureCache(1, 2, "adams_bashforth")
    for u in (0, 4, 8):
        cache.refresh(u, [np.array([a + b * u])])
    np.testing.assert_allclose(cache.forecast(11, 0), [a + b * 11], rtol=1e-13)
    # F(u) = u^2 at u = 0, 4, 8, k = 1: slopes 12 and 4 -> AB2 gives 64 + 1 * (3/2 * 12 - 1/2 * 4) = 80, Eq. 2 gives 77
    ab = core.FeatureCache(1, 2, "adams_bashforth"); ty = core.FeatureCache(1, 2, "taylor")
    for u in (0, 4, 8):
        ab.refresh(u, [np.array([float(u * u)])]); ty.refresh(u, [np.array([float(u * u)])])
    assert ab.forecast(9, 0)[0] == 80.0 and ty.forecast(9, 0)[0] == 77.0
    assert core.forecast_coefficients("adams_bashforth", 9, [8, 4, 0], 2) == [1.0, 1.0, 2.0]
    assert core.forecast_coefficients("adams_bashforth", 9, [8], 0) == [1.0]


# --- raw-feature ring layout of the cache -----------------------------------------------------


@pytest.mark.parametrize("mode", ["taylor", "newton", "adams_bashforth"])
@pytest.mark.parametrize("m", [0, 1, 2, 3, 4])
def test_ring_layout_gives_the_forecasts_of_the_difference_layout(mode, m):
    """Irregular reference steps, more of them than the ring keeps, forecasts asked for during the
    warm-up too: the two layouts agree to rounding when nothing is rounded for storage."""
    rng = np.random.default_rng(11 * m + len(mode))
    steps = [0, 3, 4, 9, 11, 16, 17, 22]
    diff = core.FeatureCache(2, m, mode); ring = core.make_cache("ring", 2, m, mode)
    for n, s in enumerate(steps):
        f = [rng.standard_normal((3, 4)), rng.standard_normal((3, 4))]
        diff.refresh(s, f); ring.refresh(s, f)
        assert ring.refs == diff.refs and ring.order_available == diff.order_available
        assert len(ring.F[0]) == min(m + 1, n + 1)
        for k in (1, 2, 4):
            for slot in (0, 1):
                np.testing.assert_allclose(ring.forecast(s + k, slot), diff.forecast(s + k, slot), rtol=1e-10, atol=1e-10)


def test_ring_layout_uniform_grid_is_eq2_written_out():
    m, N = 2, 5
    rng = np.random.default_rng(0)
    raw = [rng.standard_normal(7) for _ in range(5)]
    ring = core.make_cache("ring", 1, m, "taylor")
    for j, f in enumerate(raw):
        ring.refresh(j * N, [f])
    for k in range(1, N):
        np.testing.assert_allclose(ring.forecast(ring.refs[0] + k, 0), core.taylor_forecast_eq2(raw[::-1], N, k, m),
                                   rtol=1e-11, atol=1e-11)


def test_ring_layout_newton_reproduces_polynomials_and_rounds_features_only():
    # degree-3 polynomial sampled at irregular steps: order 3 divided differences extrapolate it exactly
    poly = lambda u: np.array([0.5 * u ** 3 - 2.0 * u ** 2 + u - 7.0, u ** 2])
    ring = core.make_cache("ring", 1, 3, "newton")
    for s in (1, 2, 5, 7, 12):
        ring.refresh(s, [poly(float(s))])
    np.testing.assert_allclose(ring.forecast(15, 0), poly(15.0), rtol=1e-12)
    # storage rounding applies to the features (and to nothing else)
    rb = core.make_cache("ring", 1, 2, "taylor", "bf16")
    f = np.array([1.2345678, -3.3333333])
    rb.refresh(0, [f]); rb.refresh(2, [2 * f])
    from speca_inputs import round_to_bf16
    assert np.array_equal(rb.F[0][0], round_to_bf16(2 * f).astype(np.float64))
    assert np.array_equal(rb.F[0][1], round_to_bf16(f).astype(np.float64))
    a, b = rb.F[0][0], rb.F[0][1]
    np.testing.assert_allclose(rb.forecast(3, 0), a + 0.5 * (a - b), rtol=1e-15)
    with pytest.raises(ValueError):
        core.make_cache("rings", 1, 1)
