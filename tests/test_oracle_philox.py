"""Pins for the oracle's noise stream (Philox4x32-10, Salmon et al. SC'11;
arXiv 2206.11357 Alg. 1 needs per-tensor seeds that replay exactly; assumption
B1 needs element-wise uncorrelated rounding).

The C oracle is checked against a second implementation written here with
Python's unbounded integers (no shared code, different word handling), and
against what a uniform, independent stream must satisfy.
"""
import numpy as np

import oracle

MASK = 0xFFFFFFFF


def philox_py(ctr, key, rounds=10):
    """Big-integer Philox-4x32: S-box = multiply, split the 64-bit product."""
    c = [int(v) for v in ctr]
    k = [int(v) for v in key]
    for _ in range(rounds):
        prod_a = 0xD2511F53 * c[0]
        prod_b = 0xCD9E8D57 * c[2]
        c = [((prod_b >> 32) ^ c[1] ^ k[0]) & MASK,
             prod_b & MASK,
             ((prod_a >> 32) ^ c[3] ^ k[1]) & MASK,
             prod_a & MASK]
        k = [(k[0] + 0x9E3779B9) & MASK, (k[1] + 0xBB67AE85) & MASK]
    return c


def noise_py(seed, i):
    blk = i // 8
    w = philox_py([blk & MASK, (blk >> 32) & MASK, 0, 0], [seed & MASK, (seed >> 32) & MASK])
    j = i % 8
    r16 = (w[j // 2] >> (16 * (j % 2))) & 0xFFFF
    return (r16 + 0.5) / 65536.0


def test_block_function_matches_bigint_implementation():
    rng = np.random.default_rng(7)
    cases = [([0, 0, 0, 0], [0, 0]), ([MASK] * 4, [MASK] * 2), ([1, 0, 0, 0], [0, 0]),
             ([0, 1, 0, 0], [0, 0]), ([0, 0, 1, 0], [0, 0]), ([0, 0, 0, 1], [0, 0]),
             ([0, 0, 0, 0], [1, 0]), ([0, 0, 0, 0], [0, 1])]
    cases += [(rng.integers(0, 2**32, 4).tolist(), rng.integers(0, 2**32, 2).tolist())
              for _ in range(200)]
    for ctr, key in cases:
        assert oracle.philox4x32_10(ctr, key).tolist() == philox_py(ctr, key), (ctr, key)


def test_each_input_word_changes_the_output():
    base = oracle.philox4x32_10([0, 0, 0, 0], [0, 0])
    seen = {tuple(base.tolist())}
    for pos in range(6):
        ctr = [0, 0, 0, 0]
        key = [0, 0]
        (ctr if pos < 4 else key)[pos % 4 if pos < 4 else pos - 4] = 1
        out = tuple(oracle.philox4x32_10(ctr, key).tolist())
        assert out not in seen
        seen.add(out)
        # avalanche: roughly half of the 128 output bits flip
        flips = sum(bin(a ^ b).count("1") for a, b in zip(out, base.tolist()))
        assert 30 <= flips <= 98


def test_noise_keying_slots_and_value_map():
    # seeds and indices that exercise both key words and both counter words
    for seed in (0, 1, 0xFFFFFFFF, 1 << 32, 0x0123456789ABCDEF, 2**64 - 1):
        for i in (0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 255, 256, 2**32 * 8 - 1, 2**32 * 8,
                  2**32 * 8 + 5, 2**40 + 3):
            assert oracle.noise(seed, i) == np.float32(noise_py(seed, i)), (seed, i)
    u = oracle.noise_array(3, 4096)
    assert u.min() >= 2.0**-17 and u.max() <= 1 - 2.0**-17
    # u*65536 - 0.5 is an integer in [0, 65535]
    r = u.astype(np.float64) * 65536 - 0.5
    assert np.all(r == np.round(r))


def test_eight_elements_share_one_block_and_use_all_of_it():
    seed = 99
    w = philox_py([5, 0, 0, 0], [seed, 0])
    got = [int(oracle.noise(seed, 40 + j) * 65536 - 0.5) for j in range(8)]
    halves = []
    for word in w:
        halves += [word & 0xFFFF, word >> 16]
    assert got == halves


def test_replay_and_seed_separation():
    a = oracle.noise_array(11, 2048)
    b = oracle.noise_array(11, 2048)
    c = oracle.noise_array(12, 2048)
    assert np.array_equal(a, b)
    assert (a == c).mean() < 0.01
    # offset replay: the stream is a pure function of (seed, i)
    assert np.array_equal(oracle.noise_array(11, 100, start=777), oracle.noise_array(11, 900)[777:877])


def test_uniformity_chi_square_and_correlations():
    n = 1 << 16
    u = np.concatenate([oracle.noise_array(s, n // 4) for s in (0, 1, 2, 3)]).astype(np.float64)
    counts = np.bincount((u * 256).astype(int), minlength=256)
    chi2 = ((counts - n / 256) ** 2 / (n / 256)).sum()
    # 255 dof: mean 255, sd 22.6; 6 sd is a one-in-a-billion bound
    assert chi2 < 255 + 6 * 22.6
    assert abs(u.mean() - 0.5) < 6 * (1 / 12) ** 0.5 / n ** 0.5
    v = u - 0.5
    for lag in (1, 2, 3, 7, 8):       # within a block and across blocks (B1)
        r = (v[:-lag] * v[lag:]).mean() / v.var()
        assert abs(r) < 6 / n ** 0.5, (lag, r)
    # same index, neighbouring seeds
    a = oracle.noise_array(100, 8192).astype(np.float64) - 0.5
    b = oracle.noise_array(101, 8192).astype(np.float64) - 0.5
    assert abs((a * b).mean() / a.var()) < 6 / 8192 ** 0.5
