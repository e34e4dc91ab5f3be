"""CPU-side checks of the C-ABI library: it loads, exports every symbol the
header declares, and its host-only entry points (sizes, argument checks, bit
allocator) agree with the oracle.  No kernel is launched here."""
import ctypes
import os
import re
import sys

import numpy as np
import pytest

import oracle
import paper_2206_11357_amd as gact

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gact.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gact_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(gact.EXPORTS)
    lib = ctypes.CDLL(gact._build.LIB)
    for name in names:
        assert getattr(lib, name) is not None


def test_bounded_copy_rejects_bad_arguments_without_a_launch():
    lib = gact.lib
    buf = (ctypes.c_char * 4096)()
    p16 = (ctypes.addressof(buf) + 15) // 16 * 16
    assert lib.gact_copy_bounded(p16, p16 + 1024, 0, 16, None) == gact.GACT_OK            # nothing to do
    assert lib.gact_copy_bounded(p16, p16 + 1024, 64, 0, None) == gact.GACT_E_ARG
    assert lib.gact_copy_bounded(p16, p16 + 1024, 64, 1025, None) == gact.GACT_E_ARG
    assert lib.gact_copy_bounded(None, p16, 64, 16, None) == gact.GACT_E_ARG
    assert lib.gact_copy_bounded(p16 + 8, p16 + 1024, 64, 16, None) == gact.GACT_E_ARG    # misaligned
    assert lib.gact_copy_bounded(p16, p16 + 1024, 64, 16, None) == gact.GACT_E_ARG        # pageable host memory


def test_size_helpers_match_the_oracle():
    for n in (0, 1, 7, 8, 31, 32, 127, 128, 129, 1000, 2048, 1 << 20, (1 << 33) + 5):
        for bits in (1, 2, 4, 8):
            assert gact.gact_packed_bytes(n, bits) == oracle.packed_bytes(n, bits)
        for G in (32, 96, 128, 256, 1024):
            assert gact.gact_num_groups(n, G) == oracle.num_groups(n, G)
    assert gact.gact_packed_bytes(-1, 2) == 0 and gact.gact_num_groups(-1, 32) == 0
    assert gact.gact_multi_workspace_bytes(0) == 0
    assert gact.gact_multi_workspace_bytes(400) >= 400 * 56 + 401 * 4


def test_argument_errors_are_reported_before_any_launch():
    lib = gact.lib
    buf = (ctypes.c_char * 4096)()
    p = ctypes.addressof(buf)
    p16 = (p + 15) // 16 * 16
    cases = [
        (dict(bits=3), gact.GACT_E_BITS), (dict(bits=0), gact.GACT_E_BITS),
        (dict(G=0), gact.GACT_E_GROUP), (dict(G=48), gact.GACT_E_GROUP),
        (dict(G=2048), gact.GACT_E_GROUP), (dict(n=-1), gact.GACT_E_ARG),
        (dict(dt=7), gact.GACT_E_ARG), (dict(x=0), gact.GACT_E_ARG),
        (dict(x=p16 + 4), gact.GACT_E_ARG), (dict(packed=0), gact.GACT_E_ARG),
        (dict(gmin=0), gact.GACT_E_ARG), (dict(gscale=p16 + 2), gact.GACT_E_ARG),
    ]
    for over, want in cases:
        a = dict(x=p16, dt=0, n=64, G=32, bits=2, packed=p16 + 1024, gmin=p16 + 2048, gscale=p16 + 3072)
        a.update(over)
        rc = lib.gact_compress(a["x"], a["dt"], a["n"], a["G"], a["bits"], 0, a["packed"],
                               a["gmin"], a["gscale"], None)
        assert rc == want, (over, rc)
        rc = lib.gact_decompress(a["packed"], a["gmin"], a["gscale"], a["n"], a["G"], a["bits"],
                                 a["x"], a["dt"], None)
        assert rc == want, (over, rc)
        rc = lib.gact_compress_footprint(a["x"], a["dt"], a["n"], a["G"], a["bits"], 0, a["packed"],
                                         a["gmin"], a["gscale"], 4, p16 + 3584, p16 + 3328, 64, None)
        assert rc == want, (over, rc)
    # the fused call's own arguments: sample count, footprint pointer, workspace
    ok = dict(x=p16, dt=0, n=64, G=32, bits=2, packed=p16 + 1024, gmin=p16 + 2048, gscale=p16 + 3072)
    fused = lambda ns, fp, ws, wsb: lib.gact_compress_footprint(
        ok["x"], ok["dt"], ok["n"], ok["G"], ok["bits"], 0, ok["packed"], ok["gmin"], ok["gscale"],
        ns, fp, ws, wsb, None)
    assert fused(-1, p16 + 3584, p16 + 3328, 64) == gact.GACT_E_ARG
    assert fused(32769, p16 + 3584, p16 + 3328, 64) == gact.GACT_E_ARG
    assert fused(4, 0, p16 + 3328, 64) == gact.GACT_E_ARG
    assert fused(4, p16 + 3584 + 4, p16 + 3328, 64) == gact.GACT_E_ARG                   # misaligned
    assert fused(4, p16 + 3584, 0, 64) == gact.GACT_E_ARG                                # no workspace
    assert fused(4, p16 + 3584, p16 + 3328, 4) == gact.GACT_E_ARG                        # too small
    assert gact.gact_compress_footprint_workspace_bytes(64, 32) == 8
    assert gact.gact_compress_footprint_workspace_bytes(2049, 256) == 16
    assert gact.gact_compress_footprint_workspace_bytes(63 * 32 + 1, 96) == 16           # 63 lanes per tile
    assert gact.gact_compress_footprint_workspace_bytes(0, 256) == 0
    assert gact.gact_compress_footprint_workspace_bytes(100, 48) == 0
    # n == 0 succeeds without touching anything
    assert lib.gact_compress(None, 0, 0, 32, 2, 0, None, None, None, None) == gact.GACT_OK
    assert lib.gact_decompress(None, None, None, 0, 32, 2, None, 0, None) == gact.GACT_OK
    # multi: checks run per descriptor, before the workspace is used
    d = (gact.TensorDesc * 2)()
    for k in range(2):
        d[k].x = p16; d[k].packed = p16 + 1024; d[k].gmin = p16 + 2048; d[k].gscale = p16 + 3072
        d[k].y = p16; d[k].n = 64; d[k].bits = 2; d[k].dtype = 0
    addr = ctypes.addressof(d)
    assert lib.gact_compress_multi(addr, -1, 32, None, 0, None) == gact.GACT_E_ARG
    assert lib.gact_compress_multi(addr, 2, 40, None, 0, None) == gact.GACT_E_GROUP
    assert lib.gact_compress_multi(addr, 0, 32, None, 0, None) == gact.GACT_OK
    assert lib.gact_compress_multi(addr, 2, 32, None, 0, None) == gact.GACT_E_ARG       # no workspace
    assert lib.gact_compress_multi(addr, 2, 32, p16, 8, None) == gact.GACT_E_ARG        # too small
    for bad in (4, -8, 8 << 48):                         # shard offsets: multiples of 8 in [0, 2^51)
        d[1].index_base = bad
        assert lib.gact_compress_multi(addr, 2, 32, p16, 4096, None) == gact.GACT_E_ARG, bad
    d[1].index_base = 0
    d[1].bits = 5
    assert lib.gact_decompress_multi(addr, 2, 32, p16, 4096, None) == gact.GACT_E_BITS
    d[1].bits = 2; d[0].n = 0; d[1].n = 0
    assert lib.gact_decompress_multi(addr, 2, 32, None, 0, None) == gact.GACT_OK       # nothing to do
    assert "bits" in gact.error_string(gact.GACT_E_BITS)
    assert "captur" in gact.error_string(gact.GACT_E_CAPTURE)


@pytest.mark.parametrize("seed", range(60))
def test_bit_allocator_is_identical_to_the_oracle(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(0, 80))
    c = rng.lognormal(0, 2, L).astype(np.float32)
    if L and seed % 3 == 0:
        c[rng.integers(0, L, max(L // 4, 1))] = c[0]          # ties
    if L and seed % 4 == 0:
        c[rng.integers(0, L, max(L // 5, 1))] = 0.0
    D = (rng.integers(0, 4000, L) * 32).astype(np.int64)
    if L and seed % 5 == 0:
        D[:] = D[0] if D[0] > 0 else 1024                     # equal sizes: many equal keys
    avg = float(rng.choice([1.0, 1.5, 2.0, 3.0, 4.0, 8.0, rng.uniform(1, 8)]))
    got = gact.gact_allocate_bits(c, D, avg)
    want = oracle.allocate_bits(c, D, avg)
    assert np.array_equal(got, want)
    assert int((got.astype(np.int64) * D).sum()) <= int(np.floor(avg * D.sum()))


def test_bit_allocator_on_the_large_mixed_set_and_its_errors():
    import synthetic_inputs as syn
    specs = syn.vit_large_set()
    c = syn.lognormal_sensitivities(len(specs), 5999)
    D = np.array([s.numel for s in specs], dtype=np.int64)
    got = gact.gact_allocate_bits(c, D, 3.0)
    assert np.array_equal(got, oracle.allocate_bits(c, D, 3.0))
    assert set(got.tolist()) <= {1, 2, 4, 8}
    for cc, dd, avg, code in (([1.0], [10], 0.99, gact.GACT_E_BUDGET),
                              ([1.0], [10], float("nan"), gact.GACT_E_BUDGET),
                              ([-1.0], [10], 2.0, gact.GACT_E_ARG),
                              ([float("inf")], [10], 2.0, gact.GACT_E_ARG),
                              ([float("nan")], [10], 2.0, gact.GACT_E_ARG),
                              ([1.0], [-1], 2.0, gact.GACT_E_ARG)):
        with pytest.raises(gact.GactError) as e:
            gact.gact_allocate_bits(cc, dd, avg)
        assert e.value.code == code


def test_variance_alert_matches_the_oracle_and_reports_errors():
    rng = np.random.default_rng(4)
    for _ in range(50):
        L = int(rng.integers(1, 40))
        c = rng.lognormal(0, 2, L).astype(np.float32)
        bits = rng.choice([1, 2, 4, 8], L).astype(np.int32)
        gv = float(rng.uniform(0.1, 100))
        alert, ratio = gact.gact_variance_alert(c, bits, gv, 1.0)
        want = oracle.variance_ratio(c, bits, gv)
        assert ratio == pytest.approx(want, rel=1e-12) and alert == (want > 1.0)
    assert gact.gact_variance_alert([], [], 1.0, 0.5) == (False, 0.0)
    for c, b, gv, code in (([1.0], [3], 1.0, gact.GACT_E_BITS), ([-1.0], [2], 1.0, gact.GACT_E_ARG),
                           ([1.0], [2], 0.0, gact.GACT_E_ARG), ([float("nan")], [2], 1.0, gact.GACT_E_ARG)):
        with pytest.raises(gact.GactError) as e:
            gact.gact_variance_alert(c, b, gv, 1.0)
        assert e.value.code == code
    assert gact.gact_reduce_workspace_bytes(0, 0) >= 16
    assert gact.gact_reduce_workspace_bytes(3, 10000) >= 3 * 32 + 16 + 2 * 8 * (10000 // 4096 + 3)


def test_variance_alert_takes_the_allocator_s_uncompressed_level():
    """Sec. 6.1 keeps the most sensitive tensors at 32 bits; the alert of Sec. 4.2 must accept exactly
    what gact_allocate_bits_levels hands out."""
    rng = np.random.default_rng(9)
    c = rng.lognormal(0, 3, 24).astype(np.float32)
    numel = rng.integers(1000, 100000, 24).astype(np.int64)
    bits = gact.gact_allocate_bits_levels(c, numel, 6.0, [1, 2, 4, 8, 32])
    assert (bits == 32).any() and (bits < 32).any()
    alert, ratio = gact.gact_variance_alert(c, bits, 2.0, 1e-3)
    assert ratio == pytest.approx(oracle.variance_ratio(c, bits, 2.0), rel=1e-12)
    # closed form, S(b) = (2^b - 1)^-2 of Sec. 4.1 in exact rationals
    from fractions import Fraction
    exact = sum(Fraction(float(cl)) / (2 ** int(b) - 1) ** 2 for cl, b in zip(c, bits)) / 2
    assert ratio == pytest.approx(float(exact), rel=1e-12)
    assert alert == (float(exact) > 1e-3)


@pytest.mark.parametrize("seed", range(40))
def test_level_set_allocator_is_identical_to_the_oracle(seed):
    rng = np.random.default_rng(1000 + seed)
    L = int(rng.integers(0, 60))
    levels = [(1, 2, 4, 8, 32), (2, 4, 8, 32), (4, 32), (1, 2, 4, 8), (8,), (1, 32)][seed % 6]
    c = rng.lognormal(0, 3, L).astype(np.float32)
    if L and seed % 3 == 0:
        c[rng.integers(0, L, max(L // 3, 1))] = c[0]
    D = (rng.integers(0, 4000, L) * 32).astype(np.int64)
    avg = float(rng.uniform(levels[0], levels[-1] + 1))
    got = gact.gact_allocate_bits_levels(c, D, avg, levels)
    assert np.array_equal(got, oracle.allocate_bits_levels(c, D, avg, levels))


def test_level_set_allocator_errors():
    c, D = [1.0, 2.0], [64, 64]
    for levels, avg, code in (((1, 3), 2.0, gact.GACT_E_BITS), ((2, 1), 2.0, gact.GACT_E_BITS),
                              ((1, 2, 4, 8, 16), 2.0, gact.GACT_E_BITS), ((2, 4), 1.5, gact.GACT_E_BUDGET),
                              ((), 2.0, gact.GACT_E_ARG)):
        with pytest.raises(gact.GactError) as e:
            gact.gact_allocate_bits_levels(c, D, avg, levels)
        assert e.value.code == code


def test_bench_refuses_more_than_one_gpu():
    """The path has no cross-GPU step; bench.py says so instead of running."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
