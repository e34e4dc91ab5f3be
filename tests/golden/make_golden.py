#!/usr/bin/env python3
"""Writes tests/golden/oracle_digests.txt: SHA-256 digests of what the CPU oracle
produces on a few seeded cases, so that a later change to the oracle's
arithmetic, to the noise stream or to the input generators cannot go unnoticed.

Calls only `oracle/` and the seeded input generators; nothing here comes from
the HIP path.  The paper (arXiv 2206.11357) prints no worked numeric example,
so these are frozen oracle outputs, not published values: they pin
reproducibility, the oracle's correctness is pinned by the property tests.

Run from the repository root:  python tests/golden/make_golden.py
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle                      # noqa: E402
import synthetic_inputs as syn     # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_digests.txt")


def sha(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def codec_cases():
    """(name, x, group_size, bits, seed); bf16 inputs as uint16 bit patterns.
    Only the value laws drawn with numpy alone, so that the inputs do not depend
    on a math library's exp or erf."""
    c1 = syn.config1()
    yield "config1_f32_n1048576_G256_b2_seed0", c1["x"], c1["group_size"], c1["bits"], c1["seed"]
    yield ("bf16_n70001_G128_b4", syn.f32_to_bf16_bits(syn.draw_numpy(syn.NORMAL, 70001, 11)), 128, 4, 12345)
    yield "f32_n8193_G96_b8_seed_above_2p63", syn.draw_numpy(syn.RELU, 8193, 12), 96, 8, 2**63 + 5
    yield "f32_n100000_G1024_b1", syn.draw_numpy(syn.OUTLIER, 100000, 13), 1024, 1, 7
    yield ("bf16_n49152_G256_b2", syn.f32_to_bf16_bits(syn.draw_numpy(syn.RELU, 49152, 14)), 256, 2, 3)


def lines():
    yield "# written by tests/golden/make_golden.py from oracle/ (CPU); SHA-256 of the raw little-endian arrays"
    for name, x, G, b, seed in codec_cases():
        p, mn, sc = oracle.compress(x, G, b, seed)
        dt = oracle.BF16 if x.dtype == np.uint16 else oracle.F32
        y = oracle.decompress(p, mn, sc, x.size, G, b, dt)
        yield "%s input=%s packed=%s gmin=%s gscale=%s dequantised=%s first_packed_bytes=%s" % (
            name, sha(x), sha(p), sha(mn), sha(sc), sha(y), p[:16].tobytes().hex())
    numel = np.array([s.numel for s in syn.vit_large_set()], dtype=np.int64)
    c = syn.lognormal_sensitivities(len(numel), 5999)
    bits = oracle.allocate_bits(c, numel, 3.0)
    yield "allocator_vit400_avg3 sensitivities=%s bits=%s histogram_1_2_4_8=%s" % (
        sha(c), sha(bits.astype(np.int32)), ",".join(str(int((bits == k).sum())) for k in (1, 2, 4, 8)))
    yield "philox_counter_0_1_2_3_key_4_5 words=%s" % ",".join(
        "%08x" % int(w) for w in oracle.philox4x32_10([0, 1, 2, 3], [4, 5]))
    # three more blocks of the generator: counter and key all zero, all ones, and the hexadecimal
    # digits of pi (the inputs for which the generator's authors publish known answers)
    ones = 0xFFFFFFFF
    for name, ctr, key in (
        ("philox_counter_zero_key_zero", [0, 0, 0, 0], [0, 0]),
        ("philox_counter_ones_key_ones", [ones] * 4, [ones] * 2),
        ("philox_counter_pi_key_pi", [0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344], [0xA4093822, 0x299F31D0]),
    ):
        yield "%s words=%s" % (name, ",".join("%08x" % int(w) for w in oracle.philox4x32_10(ctr, key)))


if __name__ == "__main__":
    text = "\n".join(lines()) + "\n"
    with open(OUT, "w") as f:
        f.write(text)
    sys.stdout.write(text)
