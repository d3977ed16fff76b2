"""CPU-side checks of the library: it loads, exports every symbol the header declares,
and its host logic (coefficients, divisors, thresholds, the per-sample schedule state
machine) agrees with the oracle.  No compute call touches a GPU here."""
import os
import re

import numpy as np
import pytest

from oracle import speca_core as core

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bd():
    from paper_2509_11628_amd import binding
    binding.load_library()
    return binding


def test_library_exports_every_declared_symbol(bd):
    hdr = open(os.path.join(ROOT, "include", "speca.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(speca_[a-z_0-9]+)\s*\(", hdr))
    assert len(declared) >= 20
    lib = bd.load_library()
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared in include/speca.h but not exported"
    assert declared == set(bd.EXPORTED)


def test_struct_layouts_match_header(bd):
    import ctypes as C
    assert C.sizeof(bd.ModelDesc) == 19 * 4
    assert C.sizeof(bd.Cfg) == 8 * 4
    assert C.sizeof(bd.Profile) == 6 * 8 * 4
    assert bd.MAX_ORDER == 4 and bd.MAX_LAUNCH_ROWS == 64


@pytest.mark.parametrize("mode", ["taylor", "newton", "adams_bashforth"])
def test_coefficients_and_divisors_match_oracle(bd, mode):
    code = {"taylor": bd.COEF_TAYLOR, "newton": bd.COEF_NEWTON, "adams_bashforth": bd.COEF_ADAMS_BASHFORTH}[mode]
    rng = np.random.default_rng(0)
    for _ in range(200):
        n = int(rng.integers(1, 6))
        refs = np.sort(rng.choice(40, size=n, replace=False))[::-1].tolist()
        step = refs[0] + int(rng.integers(1, 8))
        order = int(rng.integers(0, n))
        got = bd.coefficients(code, step, refs, order)
        exp = core.forecast_coefficients(mode, step, refs, order)
        np.testing.assert_allclose(got, np.float32(exp), rtol=1e-7)
        if order >= 1:
            np.testing.assert_array_equal(bd.divisors(code, step, refs, order), np.float32(core.refresh_divisors(mode, step, refs, order)))
    with pytest.raises(bd.SpecaError):
        bd.coefficients(code, 3, [3], 0)           # step not after the reference
    with pytest.raises(bd.SpecaError):
        bd.coefficients(code, 5, [3], 1)           # order needs two references
    with pytest.raises(bd.SpecaError):
        bd.coefficients(7, 5, [3], 0)              # unknown policy


@pytest.mark.parametrize("mode", ["taylor", "newton", "adams_bashforth"])
def test_ring_weights_reproduce_the_oracle_forecast(bd, mode):
    """Ring layout: the library's per-feature weights, applied to the raw features, give the
    oracle's forecast (difference layout and ring layout, nothing rounded) for irregular
    histories of every length, and the planes rotate."""
    code = {"taylor": bd.COEF_TAYLOR, "newton": bd.COEF_NEWTON, "adams_bashforth": bd.COEF_ADAMS_BASHFORTH}[mode]
    rng = np.random.default_rng(5)
    for m in range(0, 5):
        steps = np.cumsum(rng.integers(1, 6, size=9)).tolist()
        feats = [rng.standard_normal(6) for _ in steps]
        diff = core.FeatureCache(1, m, mode); ring = core.make_cache("ring", 1, m, mode)
        for n, (s, f) in enumerate(zip(steps, feats), start=1):
            diff.refresh(s, [f]); ring.refresh(s, [f])
            for k in (1, 3):
                w, planes = bd.ring_weights(code, m, steps[:n], s + k)
                assert len(w) == min(m + 1, n)
                assert planes.tolist() == [(n - 1 - j) % (m + 1) for j in range(len(w))]      # age j sits j planes behind
                got = sum(float(w[j]) * feats[n - 1 - j] for j in range(len(w)))
                scale = sum(abs(float(w[j])) for j in range(len(w)))
                np.testing.assert_allclose(got, diff.forecast(s + k, 0), rtol=0, atol=3e-7 * scale * 4)
                np.testing.assert_allclose(got, ring.forecast(s + k, 0), rtol=0, atol=3e-7 * scale * 4)
                assert abs(float(np.sum(w)) - 1.0) < 1e-5 * scale       # constants are forecast exactly
    with pytest.raises(bd.SpecaError):
        bd.ring_weights(code, 2, [3, 3], 5)             # full steps must increase
    with pytest.raises(bd.SpecaError):
        bd.ring_weights(code, 2, [1, 3], 3)             # forecast step not after the latest full step


def test_threshold_helpers_match_oracle(bd):
    for tau0, beta, S in ((0.5, 0.05, 50), (0.1, 0.2, 50), (0.3, 0.5, 7), (1.2, 0.9, 1)):
        np.testing.assert_allclose(bd.tau_geometric(tau0, beta, S), core.tau_geometric(tau0, beta, S), rtol=2e-7)
    np.testing.assert_allclose(bd.tau_linear(0.05, 0.01, 20), core.tau_linear(0.05, 0.01, 20), rtol=2e-7)
    assert bd.tau_linear(0.3, 0.1, 1)[0] == np.float32(0.3)
    with pytest.raises(bd.SpecaError):
        bd.tau_geometric(0.1, 0.0, 5)


def _oracle_schedule(errors, tau, order, interval, warmup):
    """Schedule the oracle's rules give for one sample when the verification error at
    step s (if attempted) is errors[s]."""
    kinds, refs = [], []
    for s in range(len(tau)):
        spec = len(refs) >= 1 and (s - refs[0]) < interval and s >= warmup and tau[s] > 0
        if spec and core.accept(errors[s], tau[s]):
            kinds.append(1)
            continue
        kinds.append(2 if spec else 0)
        refs = [s] + refs[:order]
    return kinds, refs


def test_scheduler_matches_oracle_rules_on_scripted_errors(bd):
    rng = np.random.default_rng(1)
    for trial in range(30):
        B, S = 3, 40
        order, interval, warmup = int(rng.integers(0, 4)), int(rng.integers(1, 7)), int(rng.integers(1, 4))
        tau = core.tau_geometric(0.3, 0.2, S)
        if trial % 5 == 0:
            tau[10:15] = 0.0                                    # zero threshold: forced full, no attempt
        errors = rng.uniform(0, 0.4, size=(B, S)).astype(np.float32)
        sch = bd.Scheduler(B, bd.make_cfg(order=order, interval=interval, warmup_full=warmup))
        kinds = np.zeros((B, S), np.int8)
        for s in range(S):
            spec, full = sch.plan(s, float(tau[s]))
            assert sorted(spec + full) == list(range(B))
            acc = [1 if core.accept(errors[b, s], tau[s]) else 0 for b in spec]
            kinds[:, s] = sch.commit(s, acc)
        for b in range(B):
            exp_k, exp_refs = _oracle_schedule(errors[b], tau, order, interval, warmup)
            assert kinds[b].tolist() == exp_k, (trial, b)
            assert sch.refs(b) == exp_refs


def test_scheduler_fixed_patterns_and_errors(bd):
    sch = bd.Scheduler(1, bd.make_cfg(order=2, interval=4))
    ks = []
    for s in range(10):
        spec, full = sch.plan(s, 1e9)
        ks.append(int(sch.commit(s, [1] * len(spec))[0]))
    assert ks == [0, 1, 1, 1, 0, 1, 1, 1, 0, 1]             # at most N-1 speculative steps after a full one
    with pytest.raises(bd.SpecaError):
        sch.commit(11, [])                                  # commit without plan
    with pytest.raises(bd.SpecaError):
        sch.plan(3, 1.0)                                    # step not after the latest reference
    for bad in (dict(order=5), dict(interval=0), dict(warmup_full=0), dict(coef_mode=3), dict(metric=9)):
        with pytest.raises(bd.SpecaError):
            bd.Scheduler(1, bd.make_cfg(**bad))


def test_missing_library_is_an_error(tmp_path, monkeypatch):
    from paper_2509_11628_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        binding.load_library()


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2509_11628_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt, f"{f} mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            txt = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2509_11628_amd" not in txt and "ctypes" not in txt
