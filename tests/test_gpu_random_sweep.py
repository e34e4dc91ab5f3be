"""Seeded random sweep of the GPU path against the oracle: group size (any
multiple of 32 up to 1024), bit width, dtype, length (ragged tails included),
value law, seed, and for the multi-tensor calls the number of tensors, all
drawn from one fixed generator, every output byte compared.  The fixed cases of
test_gpu_parity.py name the edge cases; this adds combinations nobody thought
of.  Quantizer: arXiv 2206.11357 App. A.4, per group (Sec. 5)."""
import numpy as np
import pytest
import torch

import oracle
import synthetic_inputs as syn
from test_gpu_parity import run_case, to_device, to_host

pytestmark = pytest.mark.gpu


def draw_case(rng):
    G = int(rng.choice([32, 64, 128, 256, 512, 1024, int(rng.integers(1, 33)) * 32]))
    bits = int(rng.choice([1, 2, 4, 8]))
    n = int(rng.choice([rng.integers(1, 5000), rng.integers(5000, 300000)]))
    law = str(rng.choice([syn.NORMAL, syn.RELU, syn.OUTLIER]))
    x = syn.draw_numpy(law, n, int(rng.integers(0, 2**31)))
    if rng.integers(0, 2):
        x = syn.f32_to_bf16_bits(x)
    return x, G, bits, int(rng.integers(0, 2**63))


def test_random_single_tensor_calls(gact):
    rng = np.random.default_rng(20260611)
    for _ in range(150):
        x, G, bits, seed = draw_case(rng)
        run_case(gact, x, G, bits, seed)


def test_random_multi_tensor_launches(gact):
    """One group size per launch, everything else per tensor; table in the kernel arguments (up to
    64 tensors) and in the workspace (more)."""
    rng = np.random.default_rng(20260612)
    for L in (1, 2, 7, 33, 64, 65, 130):
        G = int(rng.choice([32, 96, 128, 256, 1024]))
        cases = []
        for _ in range(L):
            x, _, bits, seed = draw_case(rng)
            cases.append((x[: int(rng.integers(0, min(x.size, 40000) + 1))], bits, seed))
        xs = [to_device(x) if x.size else torch.empty(0, device="cuda", dtype=torch.bfloat16 if x.dtype == np.uint16
                                                    else torch.float32) for x, _, _ in cases]
        bufs = [gact.alloc_compressed(x.size, G, b, "cuda") for x, b, _ in cases]
        ys = [torch.empty_like(x) for x in xs]
        descs = gact.make_descs(xs, [b[0] for b in bufs], [b[1] for b in bufs], [b[2] for b in bufs], ys,
                                [x.size for x, _, _ in cases], [b for _, b, _ in cases], [s for _, _, s in cases],
                                [x.dtype for x in xs])
        ws = torch.empty(gact.gact_multi_workspace_bytes(L), dtype=torch.uint8, device="cuda")
        gact.gact_compress_multi(descs, L, G, ws)
        gact.gact_decompress_multi(descs, L, G, ws)
        torch.cuda.synchronize()
        for l, (x, bits, seed) in enumerate(cases):
            if x.size == 0:
                continue
            p, mn, sc = oracle.compress(x, G, bits, seed)
            assert np.array_equal(to_host(bufs[l][0])[: p.size], p), (L, l)
            assert np.array_equal(to_host(bufs[l][1]).view(np.uint32), mn.view(np.uint32)), (L, l)
            assert np.array_equal(to_host(bufs[l][2]).view(np.uint32), sc.view(np.uint32)), (L, l)
            dt = oracle.BF16 if x.dtype == np.uint16 else oracle.F32
            y = oracle.decompress(p, mn, sc, x.size, G, bits, dt)
            assert np.array_equal(to_host(ys[l]).view(np.uint16 if dt == oracle.BF16 else np.uint32),
                                  y.view(np.uint16 if dt == oracle.BF16 else np.uint32)), (L, l)
