"""Pins for the oracle's bit allocator: arXiv 2206.11357 Eq. (ilp)
(min sum_l c_l S(b_l) s.t. sum_l b_l D_l <= budget) with S(b) = (2^b-1)^-2
from assumption B2.  Expected values come from exhaustive search over all
4^L schemes and from special cases with an obvious answer."""
import itertools

import numpy as np
import pytest

import oracle

LEVELS = (1, 2, 4, 8)


def S(b):
    return 1.0 / (2 ** b - 1) ** 2


def objective(c, bits):
    return float(sum(float(ci) * S(int(bi)) for ci, bi in zip(c, bits)))


def used(D, bits):
    return int(sum(int(d) * int(b) for d, b in zip(D, bits)))


def brute_force(c, D, budget):
    best = None
    for scheme in itertools.product(LEVELS, repeat=len(c)):
        if used(D, scheme) <= budget:
            v = objective(c, scheme)
            if best is None or v < best:
                best = v
    return best


@pytest.mark.parametrize("seed", range(40))
def test_result_is_feasible_and_optimal_for_the_bits_it_spends(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(1, 7))
    c = rng.lognormal(0, 2, L).astype(np.float32)
    D = rng.integers(1, 50, L).astype(np.int64) * 32
    avg = float(rng.uniform(1.0, 8.0))
    bits = oracle.allocate_bits(c, D, avg)
    assert set(bits.tolist()) <= set(LEVELS)
    budget = int(np.floor(avg * D.sum()))
    assert used(D, bits) <= budget
    # every state the greedy descent reaches is the exact optimum of the
    # program whose budget is that state's own cost
    best = brute_force(c, D, used(D, bits))
    assert objective(c, bits) <= best * (1 + 1e-12)
    # and it stopped at the first feasible state: the step taken last was needed
    if np.any(bits < 8):
        assert any(used(D, bits) + D[l] * (LEVELS[LEVELS.index(bits[l]) + 1] - bits[l]) > budget
                   for l in range(L) if bits[l] < 8)


def test_special_budgets():
    rng = np.random.default_rng(0)
    c = rng.lognormal(0, 2, 12).astype(np.float32)
    D = rng.integers(1, 100, 12).astype(np.int64)
    assert oracle.allocate_bits(c, D, 8.0).tolist() == [8] * 12
    assert oracle.allocate_bits(c, D, 100.0).tolist() == [8] * 12
    assert oracle.allocate_bits(c, D, 1.0).tolist() == [1] * 12
    for avg in (1, 2, 4, 8):
        assert oracle.allocate_bits(np.ones(9, np.float32), np.full(9, 64), avg).tolist() == [avg] * 9


def test_more_sensitive_tensors_get_at_least_as_many_bits():
    rng = np.random.default_rng(3)
    for avg in (1.5, 2.0, 3.0, 5.0):
        c = rng.lognormal(0, 2, 30).astype(np.float32)
        D = np.full(30, 1024, np.int64)
        bits = oracle.allocate_bits(c, D, avg)
        order = np.argsort(c, kind="stable")
        assert np.all(np.diff(bits[order]) >= 0)
        assert used(D, bits) <= avg * D.sum()


def test_zero_sensitivity_drops_first_and_ties_go_to_the_lowest_index():
    c = np.array([5.0, 0.0, 5.0, 5.0], np.float32)
    D = np.full(4, 100, np.int64)
    # budget forces exactly 700 bits out of 3200: tensor 1 falls to 1 bit first
    bits = oracle.allocate_bits(c, D, (3200 - 700) / 400)
    assert bits.tolist() == [8, 1, 8, 8]
    # one more step needed: the three equal tensors tie, index 0 goes 8 -> 4
    bits = oracle.allocate_bits(c, D, (3200 - 701) / 400)
    assert bits.tolist() == [4, 1, 8, 8]


def test_empty_tensors_and_bad_arguments():
    bits = oracle.allocate_bits([1.0, 2.0, 3.0], [0, 10, 0], 2.0)
    assert bits[0] == 8 and bits[2] == 8 and bits[1] == 2
    assert oracle.allocate_bits([], [], 3.0).size == 0
    for c, D, avg in (([1.0], [10], 0.5), ([-1.0], [10], 2.0), ([float("nan")], [10], 2.0),
                      ([float("inf")], [10], 2.0), ([1.0], [-5], 2.0), ([1.0], [10], float("nan"))):
        with pytest.raises(ValueError):
            oracle.allocate_bits(c, D, avg)


def test_large_set_budget_and_cost_ordering():
    """400 tensors, LogNormal(0,2) sensitivities, average 3 bits (the mixed-set
    shape): budget met, and no pair of one-level moves improves the result at
    equal or lower cost."""
    rng = np.random.default_rng(5999)
    c = rng.lognormal(0, 2, 400).astype(np.float32)
    D = rng.choice([25821184, 103284736, 79480832, 131072, 128000], 400).astype(np.int64)
    bits = oracle.allocate_bits(c, D, 3.0)
    assert used(D, bits) <= 3.0 * D.sum()
    assert used(D, bits) > 2.9 * D.sum()
    base = objective(c, bits)
    idx = {b: k for k, b in enumerate(LEVELS)}
    gain_up = []      # (variance removed per bit, l) for a one-level upgrade
    loss_dn = []      # (variance added per bit, l) for a one-level downgrade
    for l in range(400):
        k = idx[int(bits[l])]
        if k < 3:
            hi = LEVELS[k + 1]
            gain_up.append(float(c[l]) * (S(bits[l]) - S(hi)) / (D[l] * (hi - bits[l])))
        if k > 0:
            lo = LEVELS[k - 1]
            loss_dn.append(float(c[l]) * (S(lo) - S(bits[l])) / (D[l] * (bits[l] - lo)))
    # exchange argument: the best upgrade is never worth more per bit than the
    # cheapest further downgrade costs
    assert max(gain_up) <= min(loss_dn) * (1 + 1e-9)
    assert base > 0


# ------------------------------------------------- level sets with pass-through
def S32(b):
    return 1.0 / (2.0 ** b - 1.0) ** 2


def brute_force_levels(c, D, budget, levels):
    best = None
    for scheme in itertools.product(levels, repeat=len(c)):
        if used(D, scheme) <= budget:
            v = float(sum(float(ci) * S32(b) for ci, b in zip(c, scheme)))
            if best is None or v < best:
                best = v
    return best


@pytest.mark.parametrize("seed", range(25))
def test_level_sets_with_an_uncompressed_level_are_optimal_for_their_cost(seed):
    """Level 32 = tensor left uncompressed (the paper keeps up to 32 bits for
    the most sensitive tensors, Sec. 6.1)."""
    rng = np.random.default_rng(100 + seed)
    L = int(rng.integers(1, 6))
    levels = [(1, 2, 4, 8, 32), (2, 4, 8, 32), (4, 32), (1, 2, 4, 8), (8,)][seed % 5]
    c = rng.lognormal(0, 3, L).astype(np.float32)
    D = rng.integers(1, 50, L).astype(np.int64) * 32
    avg = float(rng.uniform(levels[0], levels[-1]))
    bits = oracle.allocate_bits_levels(c, D, avg, levels)
    assert set(bits.tolist()) <= set(levels)
    assert used(D, bits) <= int(np.floor(avg * D.sum()))
    got = float(sum(float(ci) * S32(b) for ci, b in zip(c, bits)))
    best = brute_force_levels(c, D, used(D, bits), levels)
    assert got <= best * (1 + 1e-9) + 1e-30


def test_level_set_special_cases():
    c = np.array([1.0, 1e6, 1.0, 1.0], np.float32)
    D = np.full(4, 1000, np.int64)
    lv = (1, 2, 4, 8, 32)
    assert oracle.allocate_bits_levels(c, D, 32.0, lv).tolist() == [32] * 4
    assert oracle.allocate_bits_levels(c, D, 1.0, lv).tolist() == [1] * 4
    # budget for one uncompressed tensor and 8 bits elsewhere: the sensitive one keeps 32
    assert oracle.allocate_bits_levels(c, D, (32 + 3 * 8) / 4, lv).tolist() == [8, 32, 8, 8]
    # the four-level set is the default allocator
    rng = np.random.default_rng(9)
    cc = rng.lognormal(0, 2, 30).astype(np.float32)
    DD = rng.integers(1, 99, 30).astype(np.int64)
    assert np.array_equal(oracle.allocate_bits_levels(cc, DD, 3.0, (1, 2, 4, 8)), oracle.allocate_bits(cc, DD, 3.0))
    for lv_bad, avg in (((1, 3), 2.0), ((2, 1), 2.0), ((1, 1), 2.0), ((), 2.0), ((2, 4), 1.5), ((1, 2, 4, 8, 16), 2.0)):
        with pytest.raises(ValueError):
            oracle.allocate_bits_levels(cc, DD, avg, lv_bad)
