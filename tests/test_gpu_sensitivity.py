"""GPU parity of the sensitivity reduction and the running gradient statistics
(arXiv 2206.11357 Alg. 1 and the variance alert of Sec. 4.2) against the CPU
oracle.  Both sides form every term in binary64; the oracle adds them with a
compensated sum (a few ulp for any n), the GPU adds 16 terms per thread, a tree
over the block, then at most a few hundred partials per thread and a last
tree: at most ~350 roundings of 1.1e-16 on a sum of positive terms, so the bar
is 1e-12 relative.
The running mean is binary32 per element and must be bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import synthetic_inputs as syn

pytestmark = pytest.mark.gpu
REL = 1e-12


def dev(x_np):
    if x_np.dtype == np.uint16:
        return torch.from_numpy(x_np.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(x_np).cuda()


def buffers(sizes, seed, dtype):
    out = []
    for k, n in enumerate(sizes):
        x = syn.draw_numpy(syn.NORMAL, n, seed + k) if n else np.empty(0, np.float32)
        out.append(syn.f32_to_bf16_bits(x) if dtype == "bf16" and n else
                   (np.empty(0, np.uint16) if dtype == "bf16" else x))
    return out


SIZES = [1, 3, 4, 5, 4095, 4096, 4097, 8191, 8193, 100000, 0, 12345, 1 << 20, 7]


@pytest.mark.parametrize("dtype", ("f32", "bf16"))
@pytest.mark.parametrize("bits", (1, 2, 4, 8))
def test_sensitivity_matches_the_oracle(gact, dtype, bits):
    g0 = buffers(SIZES, 10, dtype)
    g1 = buffers(SIZES, 500, dtype)
    want = oracle.sensitivity(g0, g1, bits)
    a = gact.gact_sensitivity([dev(x) for x in g0], [dev(x) for x in g1], bits)
    b = gact.gact_sensitivity([dev(x) for x in g0], [dev(x) for x in g1], bits)
    torch.cuda.synchronize()
    assert a.item() == pytest.approx(want, rel=REL)
    assert a.item() == b.item()                    # fixed reduction order
    # mixed dtypes in one gradient
    if dtype == "f32":
        h0 = g0[:6] + buffers(SIZES[6:], 10, "bf16")
        h1 = g1[:6] + buffers(SIZES[6:], 500, "bf16")
        got = gact.gact_sensitivity([dev(x) for x in h0], [dev(x) for x in h1], bits).item()
        assert got == pytest.approx(oracle.sensitivity(h0, h1, bits), rel=REL)


def test_sensitivity_special_cases(gact):
    x = dev(syn.draw_numpy(syn.NORMAL, 50000, 1))
    assert gact.gact_sensitivity([x], [x], 4).item() == 0.0
    assert gact.gact_sensitivity([], [], 2).item() == 0.0
    e = torch.empty(0, device="cuda")
    assert gact.gact_sensitivity([e, e], [e, e], 2).item() == 0.0
    k = torch.arange(1, 1001, dtype=torch.float32, device="cuda")
    assert gact.gact_sensitivity([k], [torch.zeros_like(k)], 2).item() == 0.5 * (1000 * 1001 * 2001 // 6) * 9
    with pytest.raises(gact.GactError) as err:
        gact.gact_sensitivity([x], [x], 3)
    assert err.value.code == gact.GACT_E_BITS
    with pytest.raises(gact.GactError):
        gact.gact_sensitivity([x], [x], 2, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))


def test_sensitivity_on_a_model_sized_gradient(gact):
    """Parameter list shaped like BERT-large's encoder (24 x (4 x 1024^2 + 2 x 1024 x 4096))."""
    rng = np.random.default_rng(0)
    shapes = []
    for _ in range(24):
        shapes += [1024 * 1024] * 4 + [1024 * 4096] * 2 + [1024] * 6 + [4096]
    g0 = [torch.randn(n, device="cuda", generator=torch.Generator("cuda").manual_seed(i)) for i, n in enumerate(shapes)]
    g1 = [a + 0.01 * torch.randn(a.numel(), device="cuda", generator=torch.Generator("cuda").manual_seed(1000 + i))
          for i, a in enumerate(g0)]
    got = gact.gact_sensitivity(g0, g1, 2).item()
    want = oracle.sensitivity([a.cpu().numpy() for a in g0], [a.cpu().numpy() for a in g1], 2)
    assert got == pytest.approx(want, rel=REL)


@pytest.mark.parametrize("dtype", ("f32", "bf16"))
def test_running_gradient_statistics_match_the_oracle(gact, dtype):
    sizes = [1, 5, 4096, 4099, 8192 + 3, 70000, 0, 33]
    mean_h = [np.zeros(n, np.float32) for n in sizes]
    mean_d = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in sizes]
    for t in range(1, 6):
        g = buffers(sizes, 100 * t, dtype)
        sg2 = sm2 = 0.0
        for k in range(len(sizes)):
            if sizes[k]:
                a, b = oracle.grad_stats_update(g[k], mean_h[k], t)
                sg2 += a; sm2 += b
        out = gact.gact_grad_stats_update([dev(x) for x in g], mean_d, t)
        torch.cuda.synchronize()
        assert out[0].item() == pytest.approx(sg2, rel=REL)
        assert out[1].item() == pytest.approx(sm2, rel=REL)
        for k in range(len(sizes)):
            assert np.array_equal(mean_d[k].cpu().numpy().view(np.uint32), mean_h[k].view(np.uint32)), (t, k)
    with pytest.raises(gact.GactError):
        gact.gact_grad_stats_update([dev(g[0])], [mean_d[0]], 0)


def test_variance_alert_end_to_end(gact):
    """Gradient = mu + noise: the running statistics recover the noise variance
    and the alert fires exactly when V(b) exceeds the threshold share of it."""
    n, T, sigma = 1 << 16, 50, 0.1
    gen = torch.Generator("cuda").manual_seed(5)
    mu = torch.randn(n, device="cuda", generator=gen)
    mean = torch.zeros(n, device="cuda")
    second = 0.0
    for t in range(1, T + 1):
        g = mu + sigma * torch.randn(n, device="cuda", generator=gen)
        out = gact.gact_grad_stats_update([g], [mean], t)
        second += (out[0].item() - second) / t
    var = second - out[1].item()
    assert var == pytest.approx(n * sigma**2 * (T - 1) / T, rel=0.05)
    c = np.array([9.0 * var, 225.0 * var], np.float32)          # V(b) = 2 var at bits (2, 4)
    alert, ratio = gact.gact_variance_alert(c, [2, 4], var, 1.5)
    assert alert and ratio == pytest.approx(2.0, rel=1e-6)
    assert ratio == pytest.approx(oracle.variance_ratio(c, [2, 4], var), rel=1e-12)
    alert, _ = gact.gact_variance_alert(c, [8, 8], var, 1.5)
    assert not alert


@pytest.mark.parametrize("dtype", ("f32", "bf16"))
def test_footprint_matches_the_oracle(gact, dtype):
    for n in (1, 3, 7, 4095, 4097, 100001, 1 << 21):
        x = syn.draw_numpy(syn.NORMAL, n, n % 89)
        if dtype == "bf16":
            x = syn.f32_to_bf16_bits(x)
        for ns in (0, 1, 8, 33):
            want = oracle.footprint(x, ns)
            got = gact.gact_footprint(dev(x), ns).cpu().numpy()
            assert got.shape == want.shape
            # sum of terms of both signs: absolute bar from the sum of magnitudes
            mag = float(np.sum(np.abs(syn.bf16_bits_to_f32(x) if dtype == "bf16" else x).astype(np.float64)))
            assert abs(got[0] - want[0]) <= REL * mag
            assert np.array_equal(got[1:], want[1:])
    e = torch.empty(0, device="cuda")
    assert gact.gact_footprint(e, 4).cpu().numpy().tolist() == [0.0] * 5
    k = torch.arange(1, 1001, dtype=torch.float32, device="cuda")
    assert gact.gact_footprint(k, 4).cpu().numpy().tolist() == [500500.0, 1.0, 251.0, 501.0, 751.0]


@pytest.mark.parametrize("dtype", ("f32", "bf16"))
def test_compress_with_footprint_in_one_pass(gact, dtype):
    """The fused call returns gact_compress's bytes and gact_footprint's values
    (the sum in another fixed order: same bar against the oracle)."""
    cases = [(1, 32, 2), (2047, 256, 1), (2048, 256, 2), (2049, 256, 4), (70001, 128, 8), (100000, 96, 4),
             (1 << 20, 1024, 2), (5 * 2048 * 4 + 3, 64, 2)]
    for n, G, bits in cases:
        x = syn.draw_numpy(syn.RELU if n % 2 else syn.NORMAL, n, n % 97)
        if dtype == "bf16":
            x = syn.f32_to_bf16_bits(x)
        xd = dev(x)
        for ns in (0, 8):
            p, mn, sc, fp = gact.gact_compress_footprint(xd, G, bits, 1234 + n, ns)
            p0, mn0, sc0 = gact.gact_compress(xd, G, bits, 1234 + n)
            assert torch.equal(p, p0) and torch.equal(mn, mn0) and torch.equal(sc, sc0), (n, G, bits)
            p_ref, mn_ref, sc_ref = oracle.compress(x, G, bits, 1234 + n)
            assert np.array_equal(p.cpu().numpy(), p_ref)
            want = oracle.footprint(x, ns)
            got = fp.cpu().numpy()
            mag = float(np.sum(np.abs(syn.bf16_bits_to_f32(x) if dtype == "bf16" else x).astype(np.float64)))
            assert abs(got[0] - want[0]) <= REL * mag, (n, G, bits)
            assert np.array_equal(got[1:], want[1:])
    e = torch.empty(0, device="cuda")
    out = gact.gact_compress_footprint(e, 256, 2, 0, 4)
    assert out[3].cpu().numpy().tolist() == [0.0] * 5
    k = torch.arange(1, 1001, dtype=torch.float32, device="cuda")
    assert gact.gact_compress_footprint(k, 32, 4, 0, 4)[3].cpu().numpy().tolist() == [500500.0, 1.0, 251.0, 501.0, 751.0]
