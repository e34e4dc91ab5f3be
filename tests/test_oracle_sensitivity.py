"""Pins for the oracle's sensitivity reduction and variance alert (arXiv
2206.11357 Alg. 1: return 1/2 ||g0 - g1||^2 / S(b_l); Sec. 4.2: running mean of
the gradient, alert on V(b) / Var[g]; Thm. 2: V(b) <= sum_l c_l S(b_l) with
S(b) = (2^b-1)^-2).  Expected values are closed forms and statistics."""
import numpy as np
import pytest

import oracle
import synthetic_inputs as syn


def test_sensitivity_closed_forms():
    n = 1000
    k = np.arange(1, n + 1, dtype=np.float32)
    zero = np.zeros(n, np.float32)
    sum_sq = n * (n + 1) * (2 * n + 1) // 6                   # sum k^2
    for bits, inv_S in ((1, 1), (2, 9), (4, 225), (8, 65025)):
        assert oracle.sensitivity([k], [zero], bits) == 0.5 * sum_sq * inv_S
        assert oracle.sensitivity([zero], [k], bits) == 0.5 * sum_sq * inv_S     # symmetric
        assert oracle.sensitivity([k], [k], bits) == 0.0
    # constant offset: 1/2 n delta^2 / S
    a = syn.draw_numpy(syn.NORMAL, 4096, 1)
    assert oracle.sensitivity([a + np.float32(0.5)], [a], 2) == pytest.approx(0.5 * 4096 * 0.25 * 9, rel=1e-6)
    # the norm runs over all buffers of the gradient
    parts = [k[:300], k[300:301], k[301:]]
    assert oracle.sensitivity(parts, [np.zeros_like(p) for p in parts], 4) == 0.5 * sum_sq * 225
    assert oracle.sensitivity([], [], 2) == 0.0
    # bf16 buffers are read exactly
    kb = syn.f32_to_bf16_bits(np.arange(0, 256, dtype=np.float32))
    assert oracle.sensitivity([kb], [np.zeros_like(kb)], 1) == 0.5 * (255 * 256 * 511 // 6)
    with pytest.raises(ValueError):
        oracle.sensitivity([k], [zero], 3)


def test_half_squared_difference_of_two_draws_estimates_the_variance():
    """Alg. 1 replaces a variance by the empirical variance of two evaluations:
    E[1/2 ||g0 - g1||^2] = sum of per-coordinate variances."""
    rng = np.random.default_rng(0)
    n, sigma = 200000, 0.3
    mu = rng.standard_normal(n).astype(np.float32)
    g0 = (mu + sigma * rng.standard_normal(n)).astype(np.float32)
    g1 = (mu + sigma * rng.standard_normal(n)).astype(np.float32)
    est = oracle.sensitivity([g0], [g1], 1)                   # S(1) = 1
    # chi-square with n dof scaled by sigma^2: sd = sigma^2 sqrt(2n)
    assert abs(est - n * sigma**2) < 6 * sigma**2 * np.sqrt(2 * n)


def test_running_mean_is_the_arithmetic_mean_and_moments_are_sums():
    rng = np.random.default_rng(1)
    n, T = 5000, 37
    gs = [(1.5 + rng.standard_normal(n)).astype(np.float32) for _ in range(T)]
    mean = np.zeros(n, np.float32)
    for t, g in enumerate(gs, start=1):
        sg2, sm2 = oracle.grad_stats_update(g, mean, t)
        assert sg2 == pytest.approx(float(np.sum(g.astype(np.float64) ** 2)), rel=1e-12)
        assert sm2 == pytest.approx(float(np.sum(mean.astype(np.float64) ** 2)), rel=1e-12)
        if t == 1:
            assert np.array_equal(mean, g)                    # (g - 0) * 1 + 0
    want = np.mean(np.stack(gs).astype(np.float64), axis=0)
    assert np.max(np.abs(mean - want)) < 1e-5
    # a constant gradient is a fixed point
    c = np.full(64, 0.75, np.float32)
    m = c.copy()
    oracle.grad_stats_update(c, m, 9)
    assert np.array_equal(m, c)
    # bf16 gradient
    gb = syn.f32_to_bf16_bits(gs[0])
    m2 = np.zeros(n, np.float32)
    oracle.grad_stats_update(gb, m2, 1)
    assert np.array_equal(m2, syn.bf16_bits_to_f32(gb))
    with pytest.raises(ValueError):
        oracle.grad_stats_update(c, m, 0)


def test_gradient_variance_from_running_moments():
    """Var[g] = E||g||^2 - ||E g||^2 from the two returned sums."""
    rng = np.random.default_rng(2)
    n, T, sigma = 20000, 200, 0.2
    mu = rng.standard_normal(n).astype(np.float32)
    mean = np.zeros(n, np.float32)
    second = 0.0
    for t in range(1, T + 1):
        g = (mu + sigma * rng.standard_normal(n)).astype(np.float32)
        sg2, sm2 = oracle.grad_stats_update(g, mean, t)
        second += (sg2 - second) / t
    var = second - sm2
    # sample variance with T draws underestimates by (T-1)/T
    assert var == pytest.approx(n * sigma**2 * (T - 1) / T, rel=0.02)


def test_variance_ratio_closed_forms():
    c = np.array([9.0, 225.0, 65025.0, 2.0], np.float32)
    bits = np.array([2, 4, 8, 1], np.int32)
    assert oracle.variance_ratio(c, bits, 1.0) == pytest.approx(1 + 1 + 1 + 2)
    assert oracle.variance_ratio(c, bits, 10.0) == pytest.approx(0.5)
    # more bits never raise the compression variance
    lo = oracle.variance_ratio(c, [1, 1, 1, 1], 1.0)
    hi = oracle.variance_ratio(c, [8, 8, 8, 8], 1.0)
    assert hi < oracle.variance_ratio(c, bits, 1.0) < lo
    for bad in (([1.0], [3], 1.0), ([-1.0], [2], 1.0), ([1.0], [2], 0.0)):
        with pytest.raises(ValueError):
            oracle.variance_ratio(*bad)


def test_algorithm_1_on_a_linear_gradient_recovers_the_compression_variance():
    """g(Q(h)) = w * Q(h) (elementwise).  Two runs that differ only in the
    compressor's seed give E[1/2 ||g0 - g1||^2] = sum_j w_j^2 Var[Q(h)_j], and
    Var[Q(h)_j] = frac_j (1 - frac_j) step^2 <= 1/4 step^2 (Sec. 4.1)."""
    rng = np.random.default_rng(3)
    n, G, bits, pairs = 1024, 256, 2, 400
    h = syn.draw_numpy(syn.NORMAL, n, 5)
    w = rng.standard_normal(n).astype(np.float32)
    est = 0.0
    for s in range(pairs):
        ys = []
        for seed in (2 * s, 2 * s + 1):
            p, mn, sc = oracle.compress(h, G, bits, seed)
            ys.append(w * oracle.decompress(p, mn, sc, n, G, bits))
        est += oracle.sensitivity([ys[0]], [ys[1]], bits) / (2 ** bits - 1) ** 2 / pairs   # times S(b)
    _, mn, sc = oracle.compress(h, G, bits, 0)
    step = np.repeat(sc.astype(np.float64), G)
    t = (h.astype(np.float64) - np.repeat(mn.astype(np.float64), G)) / np.where(step > 0, step, 1)
    frac = t - np.floor(t)
    want = float(np.sum(w.astype(np.float64) ** 2 * frac * (1 - frac) * step ** 2))
    bound = float(np.sum(w.astype(np.float64) ** 2 * 0.25 * step ** 2))
    assert est == pytest.approx(want, rel=0.08)
    assert est <= bound


def test_footprint_closed_forms():
    """Sec. 5.2: duplicates are recognised by sampled points and the sum."""
    n = 1000
    k = np.arange(1, n + 1, dtype=np.float32)
    f = oracle.footprint(k, 4)
    assert f[0] == n * (n + 1) / 2
    assert f[1:].tolist() == [1.0, 251.0, 501.0, 751.0]          # elements 0, 250, 500, 750
    assert oracle.footprint(k, 0).tolist() == [n * (n + 1) / 2]
    assert oracle.footprint(np.zeros(0, np.float32), 3).tolist() == [0.0, 0.0, 0.0, 0.0]
    f1 = oracle.footprint(k[:7], 3)
    assert f1.tolist() == [28.0, 1.0, 3.0, 5.0]                   # floor(j*7/3) = 0, 2, 4
    kb = syn.f32_to_bf16_bits(np.arange(0, 256, dtype=np.float32))
    assert oracle.footprint(kb, 2).tolist() == [255 * 256 / 2, 0.0, 128.0]
    # cancelling terms: exact in the compensated sum
    x = np.array([1e8, 1.0, -1e8, 1.0] * 1000, np.float32)
    assert oracle.footprint(x, 0)[0] == 2000.0
    # a changed element changes the footprint's sum
    a = syn.draw_numpy(syn.NORMAL, 5000, 3)
    b = a.copy(); b[1234] += 1e-3
    assert oracle.footprint(a, 8)[0] != oracle.footprint(b, 8)[0]
