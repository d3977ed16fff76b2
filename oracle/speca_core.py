"""CPU oracle for the SpeCa forecast / cache / verification arithmetic.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, float64 NumPy restatement of
the paper's method, used to check the HIP library.  Nothing in the product path
imports it, and it imports nothing from the product path.

Notation.  The paper indexes by a diffusion timestep that decreases while
sampling; this file uses a sampling-step index ``s = 0, 1, ...`` that increases.
``refs`` is the list of steps at which a sample was fully computed, latest first
(``refs[0]`` is the paper's key timestep ``t``); forecasting step ``s`` means the
paper's ``t-k`` with ``k = s - refs[0]``.  ``m`` is the Taylor order and ``N`` the
forced full-compute interval.

Passages followed:
  * Sec. 3.3, Eq. 2 (TaylorSeer forecast) and Eq. 3 (finite differences)
  * Sec. 3.4.1, Eq. 4 (relative L2 error, eps = 1e-8)
  * Sec. 3.4.2 (sequential validation, adaptive threshold tau_t = tau0*beta^((T-t)/T))

Readings taken where the paper is silent (each is listed in the design notes):
  * irregular gaps between full steps (after a rejection) -> divided-difference
    recursion; with a uniform gap N it reduces to Eq. 3 scaled by N^-i.
  * two coefficient policies over the same cached tensors:
      "taylor": the printed Eq. 2, c_i = k^i / i!   (differences divided by last gap)
      "newton": Newton backward divided differences, c_i = prod_{j<i}(s - r_j),
                exact for polynomials of degree <= order.
  * fewer than m+1 references available -> order min(m, n_refs-1).
"""
from __future__ import annotations

import math
from typing import Callable, List, Optional, Sequence

import numpy as np

EPS_DEFAULT = 1e-8

# ----------------------------------------------------------------------------- storage rounding


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (8-bit exponent, 7-bit fraction), ties to
    even, via float32.  Models a cache stored in bf16."""
    f = np.asarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(f.shape).astype(np.float64)


def storage_rounder(dtype: Optional[str]) -> Callable[[np.ndarray], np.ndarray]:
    """Rounding applied whenever a value is stored into the cache or an
    activation buffer of the given type.  None / "f64" keeps float64."""
    if dtype in (None, "f64"):
        return lambda a: np.asarray(a, dtype=np.float64)
    if dtype == "f32":
        return lambda a: np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_round
    raise ValueError(dtype)


# ----------------------------------------------------------------------------- Eq. 3: differences


def finite_difference_eq3(features_latest_first: Sequence[np.ndarray], i: int) -> np.ndarray:
    """Eq. 3 as printed, for uniformly spaced references:
    Delta^i F(x_t) = sum_{j=0..i} (-1)^(i-j) C(i,j) F(x_{t+jN}).

    ``features_latest_first[j]`` is F at the paper's timestep t + jN, i.e. the
    j-th most recent full step."""
    acc = np.zeros_like(np.asarray(features_latest_first[0], dtype=np.float64))
    for j in range(i + 1):
        acc = acc + ((-1.0) ** (i - j)) * math.comb(i, j) * np.asarray(features_latest_first[j], dtype=np.float64)
    return acc


def refresh_divisors(mode: str, step: int, refs_old: Sequence[int], order: int) -> List[float]:
    """Divisor d_i (i = 1..order) of the difference recursion at a new full step
    ``step`` whose previous references are ``refs_old`` (latest first).
    taylor: the last gap for every i;  newton: the span step - refs_old[i-1];
    adams_bashforth: as taylor (the same stored differences, other forecast weights)."""
    if mode in ("taylor", "adams_bashforth"):
        return [float(step - refs_old[0]) for _ in range(1, order + 1)]
    if mode == "newton":
        return [float(step - refs_old[i - 1]) for i in range(1, order + 1)]
    raise ValueError(mode)


class FeatureCache:
    """Per-sample cache of one model: for every slot the feature at the latest
    full step and its divided differences up to order m (Sec. 3.3).

    ``D[slot][i]`` is the i-th difference; ``refs`` the full steps, latest first."""

    def __init__(self, n_slots: int, order: int, mode: str = "taylor", store: Optional[str] = None):
        assert order >= 0 and mode in ("taylor", "newton", "adams_bashforth")
        self.n_slots, self.m, self.mode = n_slots, order, mode
        self.round = storage_rounder(store)
        self.D: List[List[Optional[np.ndarray]]] = [[None] * (order + 1) for _ in range(n_slots)]
        self.refs: List[int] = []

    @property
    def order_available(self) -> int:
        return min(self.m, len(self.refs) - 1)

    def refresh(self, step: int, feats: Sequence[np.ndarray]) -> None:
        """Full step at ``step``: store the new feature of every slot and update
        the differences.  D0 <- F;  D^i <- (D^{i-1}_new - D^{i-1}_old) / d_i."""
        assert len(feats) == self.n_slots
        assert not self.refs or step > self.refs[0]
        o_new = min(self.m, len(self.refs))
        div = refresh_divisors(self.mode, step, self.refs, o_new) if o_new else []
        for j in range(self.n_slots):
            old = self.D[j]
            new: List[Optional[np.ndarray]] = [None] * (self.m + 1)
            new[0] = self.round(np.asarray(feats[j], dtype=np.float64))
            # the recursion runs on the unrounded new values; each is rounded once when stored
            prev_exact = np.asarray(feats[j], dtype=np.float64)
            for i in range(1, o_new + 1):
                cur = (prev_exact - old[i - 1]) / div[i - 1]
                new[i] = self.round(cur)
                prev_exact = cur
            self.D[j] = new
        self.refs = [step] + self.refs[: self.m]

    def coefficients(self, step: int) -> List[float]:
        return forecast_coefficients(self.mode, step, self.refs, self.order_available)

    def forecast(self, step: int, slot: int) -> np.ndarray:
        """Eq. 2 for one slot at ``step`` (k = step - refs[0] > 0), float64, not rounded."""
        c = self.coefficients(step)
        acc = np.zeros_like(self.D[slot][0])
        for i, ci in enumerate(c):
            acc = acc + ci * self.D[slot][i]
        return acc


class RingFeatureCache:
    """The same cache kept as raw features: for every slot the features of the last m+1 full
    steps (each rounded once to the storage type), and no differences.  The differences of
    Eq. 3 are formed when a forecast is asked for, by the recursion's own definition
        D^0_j = F_j,   D^i_j = (D^{i-1}_j - D^{i-1}_{j+1}) / d_i(j),
    where j counts references backwards from the latest and d_i(j) is the divisor the
    difference layout used when reference j was taken (taylor, adams_bashforth: the gap
    r_j - r_{j+1}; newton: r_j - r_{j+i}).  In exact arithmetic this is the forecast of
    FeatureCache; the two differ only in what is rounded to the storage type (the features
    here, the differences there).  Same interface as FeatureCache."""

    def __init__(self, n_slots: int, order: int, mode: str = "taylor", store: Optional[str] = None):
        assert order >= 0 and mode in ("taylor", "newton", "adams_bashforth")
        self.n_slots, self.m, self.mode = n_slots, order, mode
        self.round = storage_rounder(store)
        self.F: List[List[np.ndarray]] = [[] for _ in range(n_slots)]      # latest first, at most m+1 each
        self.refs: List[int] = []

    @property
    def order_available(self) -> int:
        return min(self.m, len(self.refs) - 1)

    def refresh(self, step: int, feats: Sequence[np.ndarray]) -> None:
        assert len(feats) == self.n_slots
        assert not self.refs or step > self.refs[0]
        for j in range(self.n_slots):
            self.F[j] = [self.round(np.asarray(feats[j], dtype=np.float64))] + self.F[j][: self.m]
        self.refs = [step] + self.refs[: self.m]

    def coefficients(self, step: int) -> List[float]:
        return forecast_coefficients(self.mode, step, self.refs, self.order_available)

    def differences(self, slot: int) -> List[np.ndarray]:
        """D^0 .. D^order at the latest reference, float64."""
        r, o = self.refs, self.order_available
        level = list(self.F[slot][: o + 1])                 # D^0_j for j = 0..o
        out = [level[0]]
        for i in range(1, o + 1):
            nxt = []
            for j in range(len(level) - 1):
                d = (r[j] - r[j + i]) if self.mode == "newton" else (r[j] - r[j + 1])
                nxt.append((level[j] - level[j + 1]) / float(d))
            level = nxt
            out.append(level[0])
        return out

    def forecast(self, step: int, slot: int) -> np.ndarray:
        c = self.coefficients(step)
        D = self.differences(slot)
        acc = np.zeros_like(D[0])
        for i, ci in enumerate(c):
            acc = acc + ci * D[i]
        return acc


def make_cache(layout: str, n_slots: int, order: int, mode: str = "taylor", store: Optional[str] = None):
    if layout == "differences":
        return FeatureCache(n_slots, order, mode, store)
    if layout == "ring":
        return RingFeatureCache(n_slots, order, mode, store)
    raise ValueError(layout)


def forecast_coefficients(mode: str, step: int, refs: Sequence[int], order: int) -> List[float]:
    """Weights c_i of the cached differences in the forecast for ``step``.

    taylor (Eq. 2 as printed): with k = step - refs[0] and differences already
    divided by the gap, the term Delta^i F (-k)^i / (i! N^i) in the paper's
    decreasing-timestep indexing is  k^i / i!  times the stored i-th difference.
    newton: prod_{j<i} (step - refs[j]).
    adams_bashforth (the draft-model ablation of the appendix names the predictor but prints
    no formula; this is the textbook method in backward-difference form): one explicit
    Adams step of size h = k from the latest reference,
        y_{n+1} = y_n + h * sum_{j<q} gamma_j nabla^j f_n,
    where the derivative samples f_n, f_{n-1}, ... are the successive slopes between
    references.  The cache holds them as differences: f_n = D^1 and, the stored D^{j+1}
    being nabla^j f_n divided j times by the last gap g,  nabla^j f_n = g^j D^{j+1}.
    Hence c_0 = 1 and c_i = k * gamma_{i-1} * g^{i-1}; order q uses q slopes (AB-q)."""
    assert len(refs) >= 1 and order <= len(refs) - 1
    k = step - refs[0]
    assert k > 0
    if mode == "adams_bashforth":
        g = float(refs[0] - refs[1]) if len(refs) >= 2 else 1.0
        gam = adams_bashforth_gammas(order)
        return [1.0] + [float(k) * gam[i - 1] * g ** (i - 1) for i in range(1, order + 1)]
    if mode == "taylor":
        return [float(k) ** i / math.factorial(i) for i in range(order + 1)]
    if mode == "newton":
        c, p = [], 1.0
        for i in range(order + 1):
            c.append(p)
            p *= float(step - refs[i]) if i < len(refs) else 0.0
        return c
    raise ValueError(mode)


def adams_bashforth_gammas(q: int) -> List[float]:
    """gamma_0 .. gamma_{q-1} of the Adams-Bashforth method in backward-difference form,
    gamma_j = int_0^1 C(s + j - 1, j) ds, from the classical recurrence
        gamma_m + gamma_{m-1}/2 + gamma_{m-2}/3 + ... + gamma_0/(m+1) = 1
    (1, 1/2, 5/12, 3/8, 251/720, ...)."""
    gam: List[float] = []
    for m in range(q):
        gam.append(1.0 - sum(gam[j] / (m - j + 1) for j in range(m)))
    return gam


def taylor_forecast_eq2(features_latest_first: Sequence[np.ndarray], N: int, k: int, m: int) -> np.ndarray:
    """Eq. 2 + Eq. 3 written out directly for uniformly spaced references, in the
    paper's own indexing (timestep decreases, target is t-k):
        F_pred(x_{t-k}) = F(x_t) + sum_{i=1..m} Delta^i F(x_t) / (i! N^i) * (-k)^i
    with Delta^i from Eq. 3 over F(x_{t+jN}).

    The sign convention of Eq. 3 has F(x_{t+jN}) (an EARLIER sampling step) weighted
    (-1)^(i-j); together with (-k)^i the signs cancel into a forward extrapolation:
    (-1)^i * sum_j (-1)^(i-j) C(i,j) F_j = sum_j (-1)^j C(i,j) F_j, the backward
    difference at the latest reference."""
    out = np.asarray(features_latest_first[0], dtype=np.float64).copy()
    for i in range(1, m + 1):
        out = out + finite_difference_eq3(features_latest_first, i) / (math.factorial(i) * float(N) ** i) * float(-k) ** i
    return out


# ----------------------------------------------------------------------------- Eq. 4: verification


def relative_error_sums(pred: np.ndarray, truth: np.ndarray):
    """(sum (pred-truth)^2, sum truth^2) in float64 over all elements."""
    p = np.asarray(pred, dtype=np.float64).ravel()
    t = np.asarray(truth, dtype=np.float64).ravel()
    d = p - t
    return float(np.dot(d, d)), float(np.dot(t, t))


def relative_error(pred: np.ndarray, truth: np.ndarray, eps: float = EPS_DEFAULT) -> float:
    """Eq. 4: e = ||pred - truth||_2 / (||truth||_2 + eps), float64."""
    num, den = relative_error_sums(pred, truth)
    return math.sqrt(num) / (math.sqrt(den) + eps)


def relative_error_f32(pred: np.ndarray, truth: np.ndarray, eps: float = EPS_DEFAULT) -> np.float32:
    """Eq. 4 with the final scalar arithmetic (two square roots, add, divide) in
    float32 from float64-accumulated sums: the precision in which the accept /
    reject decision is taken."""
    num, den = relative_error_sums(pred, truth)
    return np.float32(np.sqrt(np.float32(num)) / (np.sqrt(np.float32(den)) + np.float32(eps)))


def accept(e, tau) -> bool:
    """Sec. 3.4.2: a prediction is accepted iff e <= tau (compared in float32)."""
    return bool(np.float32(e) <= np.float32(tau))


# other error metrics of the paper's ablation (appendix "Choice of Error Metrics")
def relative_error_l1(pred, truth, eps: float = EPS_DEFAULT) -> float:
    p = np.asarray(pred, dtype=np.float64).ravel(); t = np.asarray(truth, dtype=np.float64).ravel()
    return float(np.sum(np.abs(p - t)) / (np.sum(np.abs(t)) + eps))


def relative_error_linf(pred, truth, eps: float = EPS_DEFAULT) -> float:
    p = np.asarray(pred, dtype=np.float64).ravel(); t = np.asarray(truth, dtype=np.float64).ravel()
    return float(np.max(np.abs(p - t)) / (np.max(np.abs(t)) + eps))


def cosine_distance(pred, truth, eps: float = EPS_DEFAULT) -> float:
    p = np.asarray(pred, dtype=np.float64).ravel(); t = np.asarray(truth, dtype=np.float64).ravel()
    return float(1.0 - np.dot(p, t) / (math.sqrt(np.dot(p, p)) * math.sqrt(np.dot(t, t)) + eps))


# ----------------------------------------------------------------------------- thresholds


def tau_geometric(tau0: float, beta: float, steps: int) -> np.ndarray:
    """Adaptive threshold of Sec. 3.4.2, tau_t = tau0 * beta^((T-t)/T), with the
    progress (T-t)/T = s/S at sampling step s.  float32 [S]."""
    s = np.arange(steps, dtype=np.float64)
    return (tau0 * beta ** (s / steps)).astype(np.float32)


def tau_linear(tau_start: float, tau_end: float, steps: int) -> np.ndarray:
    """Linear decay from tau_start at step 0 to tau_end at step S-1.  float32 [S]."""
    if steps == 1:
        return np.array([tau_start], dtype=np.float32)
    s = np.arange(steps, dtype=np.float64) / (steps - 1)
    return (tau_start + (tau_end - tau_start) * s).astype(np.float32)


def sequential_validation(errors: Sequence[float], tau: Sequence[float]):
    """Sec. 3.4.2 on a scripted error sequence e_1..e_K with thresholds tau_1..tau_K:
    accept while e_k <= tau_k; the first e_j > tau_j rejects j and everything after.
    Returns (accepted ks, rejected ks), k counted from 1."""
    A, R = [], []
    K = len(errors)
    for k in range(1, K + 1):
        if accept(errors[k - 1], tau[k - 1]):
            A.append(k)
        else:
            R = list(range(k, K + 1))
            break
    return A, R


def speedup_model(alpha: float, gamma: float, overhead_ratio: float = 0.0) -> float:
    """Sec. 3.5 / appendix speed-up bound: S = 1 / (1 - alpha (1 - gamma - C_overhead/C))."""
    return 1.0 / (1.0 - alpha * (1.0 - gamma - overhead_ratio))
