"""Pins for the oracle's adaptive keep-ratio pieces (Sec. 5: Eq. 4, Eq. 5, Eq. 7, Alg. 1, App. D):
closed forms, invariances, and library routines taken by another route.  CPU only."""
from __future__ import annotations

import math

import numpy as np
import pytest

import oracle


# ---- Eq. 4: gradient-norm sparsity ----------------------------------------------------------------

@pytest.mark.parametrize("N", [1, 8, 32, 64, 1000])
def test_equal_norms_need_the_share_itself(N):
    # n equal norms: the n largest hold n/N of the sum, so p(s) = ceil(s N)/N (s N exact in binary here)
    a = np.full(N, 3.0, np.float32)
    for s in (0.125, 0.25, 0.5, 0.75, 1.0):
        want = max(1, math.ceil(s * N)) / N
        assert oracle.sparsity_ratio(a, s) == np.float32(want)


def test_one_dominant_sample_and_all_zero():
    a = np.zeros(16, np.float32)
    a[11] = 7.0
    for s in (0.0, 0.3, 1.0):
        assert oracle.sparsity_ratio(a, s) == np.float32(1 / 16)       # one sample holds everything
    assert oracle.sparsity_ratio(np.zeros(16, np.float32), 0.9) == np.float32(1 / 16)   # never below one sample


def test_worked_example():
    a = np.array([1, 0, 4, 1, 0, 1, 0, 1], np.float32)                 # sorted: 4 1 1 1 1 0 0 0, total 8
    got = [oracle.sparsity_ratio(a, s) for s in (0.5, 0.51, 0.875, 0.9, 1.0)]
    assert got == [np.float32(v) for v in (1 / 8, 2 / 8, 4 / 8, 5 / 8, 5 / 8)]


@pytest.mark.parametrize("seed", range(5))
def test_sparsity_against_numpy_sort_and_cumsum(seed):
    rng = np.random.default_rng(seed)
    N = int(rng.integers(2, 700))
    a = np.exp(1.5 * rng.standard_normal(N)).astype(np.float32)
    a[rng.uniform(size=N) < 0.2] = 0
    prefix = np.cumsum(np.sort(a.astype(np.float64))[::-1])            # another route: library sort + cumsum
    last = 0.0
    for s in np.linspace(0.0, 1.0, 23):
        n = int(np.searchsorted(prefix, s * prefix[-1], side="left")) + 1
        n = min(max(n, 1), N)
        got = oracle.sparsity_ratio(a, float(s))
        assert got == np.float32(n) / np.float32(N)
        assert got >= last                                             # monotone in s
        last = got
    perm = rng.permutation(N)
    assert oracle.sparsity_ratio(a[perm], 0.7) == oracle.sparsity_ratio(a, 0.7)          # order of samples
    assert oracle.sparsity_ratio(a * np.float32(4.0), 0.7) == oracle.sparsity_ratio(a, 0.7)   # scale (exact x4)


# ---- App. D: running statistics of the SGD gradient ---------------------------------------------

def test_running_statistics_match_numpy_mean_and_variance():
    rng = np.random.default_rng(3)
    M, n, stride = 6, 1000, 7
    grads = [rng.standard_normal(n).astype(np.float32) * (1 + i) for i in range(M)]
    m = (n + stride - 1) // stride
    mean = np.zeros(m, np.float32)
    sq = np.zeros(m, np.float32)
    for i, g in enumerate(grads, 1):
        oracle.grad_stats_update(g, stride, i, mean, sq)
    sub = np.stack([g[::stride] for g in grads]).astype(np.float64)
    np.testing.assert_allclose(mean, sub.mean(0), rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(sq, (sub ** 2).mean(0), rtol=1e-5, atol=1e-6)
    want = ((sub - sub.mean(0)) ** 2).sum() / (M - 1)                  # Alg. 1: 1/(M-1) sum_i ||g_i - gbar||^2
    assert oracle.grad_stats_variance(mean, sq, M) == pytest.approx(want, rel=1e-4)


def test_running_statistics_are_exact_on_a_constant_and_on_small_integers():
    mean = np.zeros(4, np.float32)
    sq = np.zeros(4, np.float32)
    g = np.array([3, -2, 0, 5], np.float32)
    for i in range(1, 5):
        oracle.grad_stats_update(g, 1, i, mean, sq)
    assert np.array_equal(mean, g) and np.array_equal(sq, g * g)
    assert oracle.grad_stats_variance(mean, sq, 4) == 0.0
    mean[:] = 0
    sq[:] = 0
    oracle.grad_stats_update(np.array([1, 1, 1, 1], np.float32), 1, 1, mean, sq)
    oracle.grad_stats_update(np.array([3, 3, 3, 3], np.float32), 1, 2, mean, sq)
    assert np.array_equal(mean, np.full(4, 2, np.float32)) and np.array_equal(sq, np.full(4, 5, np.float32))
    assert oracle.grad_stats_variance(mean, sq, 2) == 4 * 2.0          # per entry: ((1-2)^2 + (3-2)^2)/(2-1) = 2


def test_strided_squared_difference():
    rng = np.random.default_rng(1)
    a = rng.standard_normal(500).astype(np.float32)
    b = rng.standard_normal(500).astype(np.float32)
    want = ((a[::9].astype(np.float64) - b[::9]) ** 2).sum()
    assert oracle.sq_diff_strided(a, b, len(a[::9]), 9) == pytest.approx(want, rel=1e-12)
    assert oracle.sq_diff_strided(a, a, 500, 1) == 0.0


# ---- Eq. 5, Eq. 4's running maximum, Eq. 7 ---------------------------------------------------------

def test_controller_moves_s_towards_the_variance_target():
    prm = oracle.ControllerParams(alpha=0.01, beta=0.95, tau_act=0.025, tau_w=0.025)
    nu = np.array([0.5, 0.5, 0.5])
    pm = np.array([0.2, 0.5, 0.4])
    pp = np.array([0.3, 0.6, 0.5])
    # activation variance above tau_act * V_s: keep more (s up), and rho comes from the s + alpha side
    s, rho, _ = oracle.controller_update(prm, 0.80, nu, V_s=100.0, V_act=3.0, V_w=[0, 0, 0], V_s_layer=[1, 1, 1],
                                         p_minus=pm, p_plus=pp)
    assert s == pytest.approx(0.81) and np.allclose(rho, [0.3, 0.6, 0.6])
    # below: keep less (s down), rho from the s - alpha side; running maximum from the input layer up
    s, rho, _ = oracle.controller_update(prm, 0.80, nu, V_s=100.0, V_act=2.0, V_w=[0, 0, 0], V_s_layer=[1, 1, 1],
                                         p_minus=pm, p_plus=pp)
    assert s == pytest.approx(0.79) and np.allclose(rho, [0.2, 0.5, 0.5])
    # equality counts as "too high" (sign(0) = +1); s never leaves [0, 1]
    s, _, _ = oracle.controller_update(prm, 1.0, nu, 100.0, 2.5, [0, 0, 0], [1, 1, 1], pm, pp)
    assert s == 1.0
    s, _, _ = oracle.controller_update(prm, 0.0, nu, 100.0, 0.0001, [0, 0, 0], [1, 1, 1], pm, pp)
    assert s == 0.0


def test_controller_raises_nu_where_the_weight_variance_is_too_high():
    prm = oracle.ControllerParams(alpha=0.01, beta=0.5, tau_act=0.025, tau_w=0.1, nu_min=0.125)
    nu = np.array([0.5, 0.5, 0.9, 0.125])
    V_s_l = np.array([10.0, 10.0, 10.0, 10.0])
    V_w = np.array([2.0, 0.5, 2.0, 0.5])                               # threshold tau_w * V_s,l = 1
    _, _, out = oracle.controller_update(prm, 0.5, nu, 1.0, 1.0, V_w, V_s_l, [0.5] * 4, [0.5] * 4)
    assert np.allclose(out, [1.0, 0.25, 1.0, 0.125])                   # x 1/beta, x beta, capped at 1, floored
    rho_in = np.array([0.9, 0.1, 0.95, 0.2])
    _, rho, _ = oracle.controller_update(prm, 0.5, nu, 1.0, 1.0, V_w, V_s_l, rho_in, rho_in)
    assert np.all(np.diff(rho) >= 0) and np.all(rho >= rho_in) and rho[0] == rho_in[0]
