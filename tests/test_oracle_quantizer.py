"""Pins for the oracle's quantizer against what arXiv 2206.11357 and the
mathematics fix (App. A.4: transform T, two-point stochastic rounding, inverse
transform; Sec. 3.2: unbiased compressor; Sec. 4.1: variance bound with
S(b) = (2^b-1)^-2, assumptions B1 and B3).

Expected values are derived here with exact rational arithmetic, numpy's
packbits or torch's CPU casts -- never with the oracle's own formulas.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import synthetic_inputs as syn

BITS = (1, 2, 4, 8)


def exact_T(x, bits):
    """T_{h,b}(h_j) = (2^b-1)(h_j - min h)/(max h - min h), exactly."""
    xs = [Fraction(float(v)) for v in x]
    mn, mx = min(xs), max(xs)
    B = 2 ** bits - 1
    return [B * (v - mn) / (mx - mn) for v in xs], mn, mx


def away_from_integer(T, eps=Fraction(1, 10000)):
    f = T - (T.numerator // T.denominator)
    return eps < f < 1 - eps


def ulp32(v):
    return float(np.spacing(np.float32(abs(v))))


# ------------------------------------------------------------ transform T
@pytest.mark.parametrize("bits", BITS)
def test_codes_are_floor_or_ceil_of_exact_transform(bits):
    rng = np.random.default_rng(bits)
    x = (rng.standard_normal(64) * 3 + 1).astype(np.float32)
    T, _, _ = exact_T(x[:32], bits)
    T2, _, _ = exact_T(x[32:], bits)
    T = T + T2
    floors = np.array([t.numerator // t.denominator for t in T])
    ok = np.array([away_from_integer(t) for t in T])
    hi_u = np.full(64, 1 - 2.0**-17, dtype=np.float32)   # largest noise: never round up
    lo_u = np.full(64, 2.0**-17, dtype=np.float32)       # smallest noise: always round up
    p_dn, _, _ = oracle.compress_with_noise(x, 32, bits, hi_u)
    p_up, _, _ = oracle.compress_with_noise(x, 32, bits, lo_u)
    q_dn = oracle.unpack_codes(p_dn, 64, bits).astype(int)
    q_up = oracle.unpack_codes(p_up, 64, bits).astype(int)
    assert ok.sum() > 40
    assert np.array_equal(q_dn[ok], floors[ok])
    assert np.array_equal(q_up[ok], floors[ok] + 1)
    # everywhere, including near-integers: within the two neighbours
    for seed in range(20):
        p, _, _ = oracle.compress(x, 32, bits, seed)
        q = oracle.unpack_codes(p, 64, bits).astype(int)
        assert np.all((q[ok] == floors[ok]) | (q[ok] == floors[ok] + 1))
        assert q.min() >= 0 and q.max() <= 2 ** bits - 1


@pytest.mark.parametrize("bits", (1, 2, 8))
def test_rounding_rule_by_enumerating_all_noise_values(bits):
    """n = 16 (one short group): feed every one of the 65,536 possible noise
    values; the number that round up is the rounding probability, exactly."""
    rng = np.random.default_rng(100 + bits)
    x = rng.standard_normal(16).astype(np.float32)
    T, _, _ = exact_T(x, bits)
    floors = np.array([t.numerator // t.denominator for t in T])
    ok = np.array([away_from_integer(t) for t in T])
    ups = np.zeros(16, dtype=np.int64)
    prev = None
    for r in range(65536):
        u = np.full(16, (r + 0.5) / 65536.0, dtype=np.float32)
        p, _, _ = oracle.compress_with_noise(x, 32, bits, u)
        q = oracle.unpack_codes(p, 16, bits).astype(int)
        if prev is not None:
            assert np.all(q <= prev)          # larger noise never rounds higher
        prev = q
        ups += (q == floors + 1)
        assert np.all((q == floors) | (q == floors + 1) | ~ok)
    B = 2 ** bits - 1
    fp_slack = 4 * B * 2.0**-24              # rounding of t in binary32
    for j, t in enumerate(T):
        if not away_from_integer(t):
            continue
        frac = float(t - floors[j])
        assert abs(ups[j] / 65536.0 - frac) <= 2.0**-17 + fp_slack, (j, ups[j], frac)


# --------------------------------------------------- unbiasedness, variance
@pytest.mark.parametrize("bits,dtype", [(1, "f32"), (2, "f32"), (4, "f32"), (2, "bf16")])
def test_unbiased_and_variance_matches_bernoulli(bits, dtype):
    S = 12000
    G = 64
    x32 = syn.draw_numpy(syn.OUTLIER, 2 * G, 31 + bits)
    x = syn.f32_to_bf16_bits(x32) if dtype == "bf16" else x32
    xv = syn.bf16_bits_to_f32(x) if dtype == "bf16" else x32
    acc = np.zeros(2 * G)
    acc2 = np.zeros(2 * G)
    for seed in range(S):
        p, mn, sc = oracle.compress(x, G, bits, seed)
        y = oracle.decompress(p, mn, sc, 2 * G, G, bits).astype(np.float64)
        acc += y
        acc2 += y * y
    step = np.repeat(sc.astype(np.float64), G)
    mean = acc / S
    var = acc2 / S - mean ** 2
    # E[Q(x)] = x : per element within 5 sigma of the mean's standard error
    sigma = step / 2
    assert np.all(np.abs(mean - xv) <= 5 * sigma / np.sqrt(S) + 1e-6 * np.abs(xv))
    z = ((mean - xv) / (sigma / np.sqrt(S) + 1e-30)).mean() * np.sqrt(2 * G)
    assert abs(z) < 5
    # Var <= 1/4 (range/(2^b-1))^2 = step^2/4
    assert np.all(var <= 0.25 * step ** 2 * 1.08)
    # and equals frac(1-frac) step^2 (two-point law)
    Tg = exact_T(xv[:G], bits)[0] + exact_T(xv[G:], bits)[0]
    frac = np.array([float(t - (t.numerator // t.denominator)) for t in Tg])
    expect = frac * (1 - frac) * step ** 2
    assert np.all(np.abs(var - expect) <= 0.08 * 0.25 * step ** 2 + 1e-12)


def test_rounding_is_uncorrelated_across_elements():
    """Assumption B1: Cov[Q(h)_i, Q(h)_j] = 0 for i != j (neighbours share a
    Philox block, so test those in particular)."""
    S = 8000
    G = 32
    x = np.linspace(0.0, 1.0, G).astype(np.float32) ** 2
    errs = np.empty((S, G))
    for seed in range(S):
        p, mn, sc = oracle.compress(x, G, 2, seed)
        errs[seed] = oracle.decompress(p, mn, sc, G, G, 2) - x
    live = errs.std(axis=0) > 1e-9
    c = np.corrcoef(errs[:, live].T)
    off = c[~np.eye(c.shape[0], dtype=bool)]
    assert np.abs(off).max() < 6 / np.sqrt(S)


@pytest.mark.parametrize("bits", BITS)
def test_error_never_exceeds_one_step(bits):
    x = syn.draw_numpy(syn.OUTLIER, 4096, 77)
    for seed in range(10):
        p, mn, sc = oracle.compress(x, 256, bits, seed)
        y = oracle.decompress(p, mn, sc, 4096, 256, bits)
        step = np.repeat(sc, 256).astype(np.float64)
        err = np.abs(y.astype(np.float64) - x)
        slack = 4 * np.spacing(np.abs(x) + np.abs(np.repeat(mn, 256)) + step.astype(np.float32))
        assert np.all(err <= step * (1 + 2.0**-20) + slack)


# ------------------------------------------------------------ exact cases
@pytest.mark.parametrize("bits", BITS)
def test_constant_and_degenerate_groups_round_trip_exactly(bits):
    G = 32
    x = np.concatenate([np.full(G, 3.25, np.float32), np.full(G, -7.0, np.float32),
                        np.zeros(G, np.float32), np.full(G, 1e-30, np.float32)])
    x[2 * G + 3] = -0.0
    x[3 * G + 1] = np.float32(1e-30) + np.float32(2.0**-110)   # range far below 2^-100
    p, mn, sc = oracle.compress(x, G, bits, 5)
    assert np.all(sc == 0) and np.all(np.signbit(sc) == False)
    assert np.all(p == 0)
    y = oracle.decompress(p, mn, sc, 4 * G, G, bits)
    assert np.array_equal(y[:2 * G], x[:2 * G])
    assert np.all(y[2 * G:3 * G] == 0) and not np.signbit(mn[2])
    assert np.all(y[3 * G:] == mn[3])


def test_negative_zero_minimum_is_stored_as_positive_zero():
    x = np.abs(syn.draw_numpy(syn.NORMAL, 64, 3))
    x[5] = -0.0
    x[40] = 0.0
    _, mn, _ = oracle.compress(x, 32, 2, 0)
    assert mn[0] == 0 and not np.signbit(mn[0])
    assert mn[1] == 0 and not np.signbit(mn[1])


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("k", (-3, 0, 5))
def test_inputs_on_the_grid_are_reproduced_for_every_seed(bits, k):
    """B3 (idempotence): h = Q(h') implies Q(h) = h.  Grid: min integer,
    range = (2^b-1) 2^k, so T is an exact integer in binary32."""
    B = 2 ** bits - 1
    rng = np.random.default_rng(bits * 10 + k + 3)
    G = 64
    j = rng.integers(0, B + 1, size=2 * G)
    j[0], j[1], j[G], j[G + 1] = 0, B, B, 0
    mn = np.repeat(np.array([-4.0, 17.0], np.float32), G)
    x = (mn + j * np.float32(2.0 ** k)).astype(np.float32)
    for seed in range(25):
        p, gmn, sc = oracle.compress(x, G, bits, seed)
        assert np.array_equal(oracle.unpack_codes(p, 2 * G, bits), j.astype(np.uint8))
        assert np.array_equal(sc, np.full(2, 2.0 ** k, np.float32))
        assert np.array_equal(oracle.decompress(p, gmn, sc, 2 * G, G, bits), x)


def test_recompressing_an_output_almost_never_changes_codes():
    x = syn.draw_numpy(syn.NORMAL, 1 << 14, 9)
    p, mn, sc = oracle.compress(x, 256, 4, 1)
    y = oracle.decompress(p, mn, sc, x.size, 256, 4)
    p2, _, _ = oracle.compress(y, 256, 4, 2)
    q, q2 = oracle.unpack_codes(p, x.size, 4), oracle.unpack_codes(p2, x.size, 4)
    # groups that use both extreme codes keep their min/range, hence their grid
    full = np.repeat((q.reshape(-1, 256).min(1) == 0) & (q.reshape(-1, 256).max(1) == 15), 256)
    assert full.mean() > 0.9
    assert (q[full] != q2[full]).mean() < 1e-3


@pytest.mark.parametrize("bits", BITS)
def test_extremes_get_the_end_codes(bits):
    B = 2 ** bits - 1
    x = syn.draw_numpy(syn.NORMAL, 2048, 21)
    g = x.reshape(-1, 256)
    lo, hi = g.argmin(1) + np.arange(8) * 256, g.argmax(1) + np.arange(8) * 256
    for seed in range(40):
        p, mn, sc = oracle.compress(x, 256, bits, seed)
        q = oracle.unpack_codes(p, 2048, bits)
        assert np.all(q[lo] == 0)
        assert np.all(q[hi] == B)
        assert q.max() <= B
        assert np.array_equal(mn, g.min(1))
        # stored step is range/(2^b-1) to one rounding
        want = (g.max(1).astype(np.float64) - g.min(1)) / B
        assert np.all(np.abs(sc - want) <= np.spacing(sc))


def test_noise_equal_to_the_fraction_does_not_round_up():
    """Strict comparison: P(up) = #{r : (r+1/2)/2^16 < frac} / 2^16, so a value
    whose fraction is exactly (r0+1/2)/2^16 rounds up for r0 noise values, and
    a zero fraction never rounds up."""
    r0 = 40000
    x = np.zeros(32, np.float32)
    x[1] = 1.0
    x[2] = (r0 + 0.5) / 65536.0               # b = 1, range 1: T(x) = x exactly
    ups = 0
    for r in (0, 1, r0 - 1, r0, r0 + 1, 65535):
        u = np.full(32, (r + 0.5) / 65536.0, np.float32)
        q = oracle.unpack_codes(oracle.compress_with_noise(x, 32, 1, u)[0], 32, 1)
        assert q[2] == (1 if r < r0 else 0), r
        assert q[0] == 0 and q[1] == 1 and np.all(q[3:] == 0)


def test_code_never_exceeds_the_top_level_when_rounding_overshoots():
    """(max-min) * fl(B/(max-min)) can land one ulp above B in binary32; the
    code must stay B even under the smallest noise value."""
    rng = np.random.default_rng(2)
    x = rng.standard_normal(400 * 32).astype(np.float32)
    u = np.full(x.size, 2.0**-17, np.float32)
    p, mn, sc = oracle.compress_with_noise(x, 32, 8, u)
    g = x.reshape(-1, 32)
    top = g.argmax(1) + np.arange(400) * 32
    t_max = (g.max(1) - g.min(1)) * (np.float32(255) / (g.max(1) - g.min(1)))
    assert (t_max > 255).sum() >= 10           # the overshoot does occur
    assert np.all(p[top] == 255)
    y = oracle.decompress(p, mn, sc, x.size, 32, 8)
    assert np.all(np.abs(y[top] - x[top]) <= 2 * np.spacing(np.abs(x[top]) + np.abs(g.min(1))))


def test_bf16_output_ties_round_to_even():
    # grid 1 + j/256, j = 0..255: every odd j is an exact bf16 tie
    x = (1.0 + np.arange(256) / 256.0).astype(np.float32)
    p, mn, sc = oracle.compress(x, 256, 8, 0)
    assert sc[0] == np.float32(2.0**-8) and mn[0] == 1.0
    y32 = oracle.decompress(p, mn, sc, 256, 256, 8, oracle.F32)
    assert np.array_equal(y32, x)
    y16 = oracle.decompress(p, mn, sc, 256, 256, 8, oracle.BF16)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(y16, want)
    # spelled out for the first ties: 1+1/256 -> 1 (even), 1+3/256 -> 1+4/256
    assert y16[1] == 0x3F80 and y16[3] == 0x3F82 and y16[5] == 0x3F82


# ------------------------------------------------------- layout and inverse
@pytest.mark.parametrize("bits", BITS)
def test_packed_layout_is_numpy_packbits_little(bits):
    n = 1000                                  # ragged: not a multiple of 8, 32 or G
    x = syn.draw_numpy(syn.NORMAL, n, 5)
    half = np.full(n, 0.5, dtype=np.float32)    # noise 1/2: round to nearest
    p, mn, sc = oracle.compress_with_noise(x, 96, bits, half)
    codes = np.empty(n, dtype=np.int64)
    for g0 in range(0, n, 96):
        T, _, _ = exact_T(x[g0:g0 + 96], bits)
        Th = [t + Fraction(1, 2) for t in T]
        assert all(away_from_integer(t) or t.denominator == 2 for t in Th)
        codes[g0:g0 + 96] = [t.numerator // t.denominator for t in Th]
    codes = np.minimum(codes, 2 ** bits - 1)
    bitplanes = ((codes[:, None] >> np.arange(bits)) & 1).astype(np.uint8).reshape(-1)
    want = np.packbits(bitplanes, bitorder="little")
    nbytes = (n * bits + 7) // 8
    assert p.size == oracle.packed_bytes(n, bits) == -(-nbytes // 16) * 16
    assert np.array_equal(p[:nbytes], want[:nbytes])
    assert np.all(p[nbytes:] == 0)
    if bits == 8:
        assert np.array_equal(p[:n], codes.astype(np.uint8))
    assert np.array_equal(oracle.unpack_codes(p, n, bits), codes.astype(np.uint8))


@pytest.mark.parametrize("bits", BITS)
def test_inverse_transform_is_min_plus_code_times_step(bits):
    n, G = 700, 128
    x = syn.draw_numpy(syn.OUTLIER, n, 8)
    p, mn, sc = oracle.compress(x, G, bits, 4)
    q = oracle.unpack_codes(p, n, bits)
    y = oracle.decompress(p, mn, sc, n, G, bits)
    for i in range(n):
        g = i // G
        exact = Fraction(float(mn[g])) + int(q[i]) * Fraction(float(sc[g]))
        prod = int(q[i]) * float(sc[g])             # exact in binary64: 8 x 24 bits
        # two roundings: product to binary32, then the sum
        assert abs(Fraction(float(y[i])) - exact) <= Fraction(ulp32(prod)) / 2 + Fraction(ulp32(y[i])) / 2
        if q[i] == 0:
            assert y[i] == mn[g]


def test_groups_are_quantized_independently():
    G, bits = 64, 2
    x = syn.draw_numpy(syn.NORMAL, 5 * G - 7, 13)
    u = np.random.default_rng(1).random(x.size, dtype=np.float32)
    p, mn, sc = oracle.compress_with_noise(x, G, bits, u)
    for g in range(5):
        sl = slice(g * G, min((g + 1) * G, x.size))
        pg, mg, sg = oracle.compress_with_noise(x[sl], G, bits, u[sl])
        nb = ((sl.stop - sl.start) * bits + 7) // 8
        assert np.array_equal(p[g * G * bits // 8: g * G * bits // 8 + nb], pg[:nb])
        assert mg[0] == mn[g] and sg[0] == sc[g]
    # a change in one group leaves the other groups' bytes alone
    x2 = x.copy()
    x2[G + 3] = 50.0
    p2, _, _ = oracle.compress_with_noise(x2, G, bits, u)
    gb = G * bits // 8
    assert np.array_equal(p[:gb], p2[:gb]) and np.array_equal(p[2 * gb:], p2[2 * gb:])
    assert not np.array_equal(p[gb:2 * gb], p2[gb:2 * gb])


def test_tail_group_uses_only_its_own_elements():
    G = 256
    x = syn.draw_numpy(syn.NORMAL, G + 5, 17)
    p, mn, sc = oracle.compress(x, G, 4, 3)
    assert mn[1] == x[G:].min()
    assert abs(sc[1] - (float(x[G:].max()) - float(x[G:].min())) / 15) <= np.spacing(sc[1])
    y = oracle.decompress(p, mn, sc, G + 5, G, 4)
    assert np.all(np.abs(y[G:] - x[G:]) <= sc[1] * 1.001)


# ------------------------------------------------------------------- bf16
@pytest.mark.parametrize("bits", (2, 8))
def test_bf16_input_is_widened_exactly_and_output_rounded_to_nearest_even(bits):
    n, G = 3000, 128
    xb = syn.f32_to_bf16_bits(syn.draw_numpy(syn.NORMAL, n, 23))
    xf = syn.bf16_bits_to_f32(xb)
    pb, mb, sb = oracle.compress(xb, G, bits, 6)
    pf, mf, sf = oracle.compress(xf, G, bits, 6)
    assert np.array_equal(pb, pf) and np.array_equal(mb, mf) and np.array_equal(sb, sf)
    y32 = oracle.decompress(pb, mb, sb, n, G, bits, oracle.F32)
    y16 = oracle.decompress(pb, mb, sb, n, G, bits, oracle.BF16)
    want = torch.from_numpy(y32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(y16, want)


# ------------------------------------------------------------ sizes, errors
def test_compression_ratio_closed_form():
    """32-bit -> 2-bit is 16x before metadata (Sec. 3.1); with two fp32 words
    per group of 256 a 4-bit code gives 8*4/(4+64/256) = 7.53x, next to the
    7.54-7.56x the paper's Table 3 prints for fixed 4 bits."""
    n = 1 << 20
    assert n * 4 / oracle.packed_bytes(n, 2) == 16.0
    total = oracle.packed_bytes(n, 4) + 8 * oracle.num_groups(n, 256)
    assert abs(n * 4 / total - 32 / (4 + 64 / 256)) < 1e-9
    assert abs(n * 4 / total - 7.53) < 0.01
    assert oracle.num_groups(1000, 256) == 4 and oracle.num_groups(1024, 256) == 4
    assert oracle.packed_bytes(0, 2) == 0 and oracle.packed_bytes(1, 1) == 16
    assert oracle.packed_bytes(129, 8) == 144


def test_bad_arguments_are_rejected():
    x = np.zeros(64, np.float32)
    for G, b in ((0, 2), (16, 2), (48, 2), (2048, 2), (64, 3), (64, 0), (64, 16)):
        with pytest.raises(ValueError):
            oracle.compress(x, G, b, 0)
    p, mn, sc = oracle.compress(np.zeros(0, np.float32), 64, 2, 0)
    assert p.size == 0 and mn.size == 0 and sc.size == 0
