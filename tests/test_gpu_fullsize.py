"""GPU parity at the full sizes of the benchmark workloads, in the launch
configuration bench.py times (bits from the allocator, one multi-tensor launch
per direction).  Three levels:
(a) whole tensors, every byte of packed codes, minima, steps and dequantised
values against the oracle: all tensors of the ResNet-50- and GCN-shaped sets,
and of the BERT-large- and ViT-shaped sets (10^10 elements, too many for the
oracle) one tensor of every distinct (shape class, bit width);
(b) for every tensor of every set, sampled runs of groups -- the first and last
tile, tile and block boundaries, and random positions -- which the oracle
computes one slice at a time from the same (seed, element index) noise;
(c) properties that hold for every group at any size: stored minimum is the
true minimum, stored step is range/(2^b-1) to one rounding, |y - x| <= step,
codes within [0, 2^b-1] (implied by the error bound), pad bytes zero.
Quantizer: arXiv 2206.11357 App. A.4 per group; sets shaped like its CNN,
transformer and GNN workloads (Sec. 6)."""
import numpy as np
import pytest
import torch

import oracle
import synthetic_inputs as syn

pytestmark = pytest.mark.gpu


def host(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def check_sampled_slices(gact, x, packed, gmin, gscale, y, n, G, bits, seed, rng, n_random):
    """Bit-exact comparison of sampled group runs with the oracle."""
    ng = (n + G - 1) // G
    run = max(2048 // G, 1) * 2                    # two wavefront tiles worth of groups
    starts = {0, max(ng - run, 0), max((8192 // G) - run // 2, 0)}
    starts |= {int(g) for g in rng.integers(0, max(ng - run, 1), n_random)}
    dt = oracle.BF16 if x.dtype == torch.bfloat16 else oracle.F32
    for g0 in sorted(starts):
        g1 = min(g0 + run, ng)
        e0, e1 = g0 * G, min(g1 * G, n)
        xs = host(x[e0:e1])
        p_ref, mn_ref, sc_ref = oracle.compress_slice(xs, G, bits, seed, e0)
        nb = ((e1 - e0) * bits + 7) // 8
        b0 = e0 * bits // 8
        assert np.array_equal(host(packed[b0:b0 + nb]), p_ref[:nb]), ("packed", g0)
        assert np.array_equal(host(gmin[g0:g1]).view(np.uint32), mn_ref.view(np.uint32)), ("gmin", g0)
        assert np.array_equal(host(gscale[g0:g1]).view(np.uint32), sc_ref.view(np.uint32)), ("gscale", g0)
        y_ref = oracle.decompress(p_ref, mn_ref, sc_ref, e1 - e0, G, bits, dt)
        y_h = host(y[e0:e1])
        if dt == oracle.F32:
            assert np.allclose(y_h, y_ref, rtol=1e-6, atol=0) and np.array_equal(y_h, y_ref), ("y", g0)
        else:
            assert np.all(np.abs(y_h.astype(np.int32) - y_ref.astype(np.int32)) <= 1)
            assert np.array_equal(y_h, y_ref), ("y", g0)


def check_properties(x, packed, gmin, gscale, y, n, G, bits):
    """Whole-tensor invariants, evaluated on the device with torch ops."""
    assert n % G == 0                              # true for every benchmark tensor
    B = float(2 ** bits - 1)
    xf = x.view(-1, G).float()
    mn = xf.amin(dim=1)
    mx = xf.amax(dim=1)
    assert torch.equal(gmin, mn + 0.0)
    want = ((mx.double() - mn.double()) / B)
    step = gscale.double()
    ulp = torch.maximum(step.abs(), torch.tensor(1e-38, device=x.device, dtype=torch.float64)) * 2.0**-23
    assert bool(((step - want).abs() <= ulp + 2.0**-100).all())
    err = (y.view(-1, G).double() - xf.double()).abs()
    # one step, plus the output rounding (bf16 output: half an ulp of |y|)
    slack = 2.0**-20 * step[:, None]
    if y.dtype == torch.bfloat16:
        slack = slack + y.view(-1, G).double().abs() * 2.0**-8
    else:
        slack = slack + (xf.double().abs() + step[:, None]) * 2.0**-22
    assert bool((err <= step[:, None] + slack).all())
    nb = (n * bits + 7) // 8
    assert packed.numel() >= nb and bool((packed[nb:(nb + 15) // 16 * 16] == 0).all())


def shape_class(spec):
    """Tensors of one set that share shape and value law: the name without layer and copy numbers."""
    return spec.name.split(".")[-1].rstrip("0123456789")


def whole_tensor_indices(specs, bits, every):
    """All tensors, or the first tensor of every distinct (shape class, bit width)."""
    if every:
        return list(range(len(specs)))
    seen, out = set(), []
    for l, (s, b) in enumerate(zip(specs, bits)):
        key = (shape_class(s), s.shape, int(b))
        if key not in seen:
            seen.add(key)
            out.append(l)
    return out


def check_whole_tensor(x, packed, gmin, gscale, y, n, G, bits, seed, name):
    """Every byte the two kernels wrote for this tensor against the oracle."""
    xh = host(x)
    p_ref, mn_ref, sc_ref = oracle.compress(xh, G, bits, seed)
    assert np.array_equal(host(gmin).view(np.uint32), mn_ref.view(np.uint32)), ("gmin", name)
    assert np.array_equal(host(gscale).view(np.uint32), sc_ref.view(np.uint32)), ("gscale", name)
    assert np.array_equal(host(packed[:p_ref.size]), p_ref), ("packed", name)
    dt = oracle.BF16 if x.dtype == torch.bfloat16 else oracle.F32
    y_ref = oracle.decompress(p_ref, mn_ref, sc_ref, n, G, bits, dt)
    y_h = host(y)
    if dt == oracle.F32:
        assert np.array_equal(y_h.view(np.uint32), y_ref.view(np.uint32)), ("y", name)     # bar: 1e-6 relative
    else:
        assert np.array_equal(y_h, y_ref), ("y", name)                                     # bar: one bf16 ulp
    return n


def run_set(gact, specs, G, avg_bits, sens_seed, n_random, uniform_bits=None, whole_every=False):
    dev = torch.device("cuda:0")
    L = len(specs)
    numel = np.array([s.numel for s in specs], dtype=np.int64)
    if uniform_bits is None:
        sens = syn.lognormal_sensitivities(L, sens_seed)
        bits = gact.gact_allocate_bits(sens, numel, avg_bits)
        assert np.array_equal(bits, oracle.allocate_bits(sens, numel, avg_bits))
        assert int((bits.astype(np.int64) * numel).sum()) <= int(np.floor(avg_bits * numel.sum()))
    else:
        bits = np.full(L, uniform_bits, dtype=np.int32)
    xs = [syn.draw_torch(s, dev) for s in specs]
    packed, gmin, gscale, ys = [], [], [], []
    for s, x, b in zip(specs, xs, bits):
        p, mn, sc = gact.alloc_compressed(s.numel, G, int(b), dev)
        p.fill_(0x5A)
        packed.append(p); gmin.append(mn); gscale.append(sc)
        ys.append(torch.empty_like(x))
    seeds = [s.seed for s in specs]
    descs = gact.make_descs(xs, packed, gmin, gscale, ys, numel, bits, seeds, [x.dtype for x in xs])
    ws = torch.empty(gact.gact_multi_workspace_bytes(L), dtype=torch.uint8, device=dev)
    gact.gact_compress_multi(descs, L, G, ws)
    gact.gact_decompress_multi(descs, L, G, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(sens_seed)
    for l in range(L):
        n, b = int(numel[l]), int(bits[l])
        check_sampled_slices(gact, xs[l], packed[l], gmin[l], gscale[l], ys[l], n, G, b, seeds[l],
                             rng, n_random)
        check_properties(xs[l], packed[l], gmin[l], gscale[l], ys[l], n, G, b)
    whole = whole_tensor_indices(specs, bits, whole_every)
    checked = sum(check_whole_tensor(xs[l], packed[l], gmin[l], gscale[l], ys[l], int(numel[l]), G, int(bits[l]),
                                     seeds[l], specs[l].name) for l in whole)
    assert checked > 0
    if not whole_every:
        classes = {(shape_class(s), s.shape) for s in specs}
        assert {(shape_class(specs[l]), specs[l].shape) for l in whole} == classes
    return bits


def test_resnet50_set_full_size(gact):
    specs = syn.resnet50_set()
    bits = run_set(gact, specs, 256, 2.0, 2999, n_random=6, whole_every=True)
    assert len(set(bits.tolist())) >= 3            # the allocator really mixes widths


@pytest.mark.parametrize("bits", (2, 4))
def test_gcn_set_full_size(gact, bits):
    run_set(gact, syn.gcn_set(), 256, None, 4000 + bits, n_random=8, uniform_bits=bits, whole_every=True)


def test_bert_large_set_full_size(gact):
    run_set(gact, syn.bert_large_set(), 256, 4.0, 3999, n_random=3)


def test_vit_large_set_full_size(gact):
    bits = run_set(gact, syn.vit_large_set(), 128, 3.0, 5999, n_random=2)
    assert set(bits.tolist()) <= {1, 2, 4, 8}


def test_single_tensor_beyond_32_bit_element_indices(gact):
    """n > 2^32: the high counter word of the noise and 64-bit addressing."""
    dev = torch.device("cuda:0")
    n = (1 << 32) + 5 * 8192 + 256
    G, bits, seed = 256, 2, (1 << 40) + 3
    x = torch.empty(n, dtype=torch.bfloat16, device=dev)
    x.normal_(generator=torch.Generator(device=dev).manual_seed(77))
    packed, gmin, gscale = gact.gact_compress(x, G, bits, seed)
    y = gact.gact_decompress(packed, gmin, gscale, n, G, bits, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    ng = n // G
    for g0 in (0, (1 << 32) // G - 8, (1 << 32) // G, ng - 16, int(rng.integers(0, ng - 16))):
        e0, e1 = g0 * G, (g0 + 16) * G
        p_ref, mn_ref, sc_ref = oracle.compress_slice(host(x[e0:e1]), G, bits, seed, e0)
        assert np.array_equal(host(packed[e0 * bits // 8: e1 * bits // 8]), p_ref[:(e1 - e0) * bits // 8])
        assert np.array_equal(host(gmin[g0:g0 + 16]), mn_ref)
        y_ref = oracle.decompress(p_ref, mn_ref, sc_ref, e1 - e0, G, bits, oracle.BF16)
        assert np.array_equal(host(y[e0:e1]), y_ref)
