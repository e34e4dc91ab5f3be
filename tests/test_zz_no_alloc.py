"""The entry point that allocates nothing, gact_compress_footprint_noalloc,
against gact_compress_footprint on the same inputs: packed codes, group minima,
steps and the footprint must be identical, on two calls in a row that share the
library's scratch area, the second on a smaller tensor."""
import ctypes

import numpy as np
import pytest
import torch

import synthetic_inputs as syn

pytestmark = pytest.mark.gpu


def device_input(dtype, n, seed):
    x_np = syn.draw_numpy(syn.OUTLIER, n, seed)
    if dtype == "bf16":
        bits = syn.f32_to_bf16_bits(x_np)
        return torch.from_numpy(bits.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(x_np).cuda()


def both_ways(gact, x, G, bits, seed, n_samples):
    n = x.numel()
    ref = gact.gact_compress_footprint(x, G, bits, seed, n_samples)
    packed, gmin, gscale = gact.alloc_compressed(n, G, bits, x.device)
    for t in (packed, gmin, gscale):
        t.view(torch.uint8).fill_(0xA5)
    fp = torch.full((1 + n_samples,), float("nan"), dtype=torch.float64, device=x.device)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    gact.gact_compress_footprint_noalloc(x, G, bits, seed, n_samples, packed, gmin, gscale, fp)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for got, want, what in zip((packed, gmin, gscale), ref[:3], ("packed", "gmin", "gscale")):
        assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), what
    assert torch.equal(fp.view(torch.int64), ref[3].view(torch.int64)), "footprint"


@pytest.mark.parametrize("dtype,G,bits", [("f32", 256, 2), ("bf16", 128, 4), ("f32", 96, 8), ("bf16", 1024, 1)])
def test_two_calls_in_a_row_match_the_workspace_call(gact, dtype, G, bits):
    big = device_input(dtype, 5 * 8192 * 11 + 1234, 71)       # several blocks and a ragged tail
    both_ways(gact, big, G, bits, seed=9, n_samples=8)
    small = device_input(dtype, 3 * 2048 + 77, 72)            # fewer tiles: stale partials lie behind its own
    both_ways(gact, small, G, bits, seed=10, n_samples=5)
    both_ways(gact, small[:0], G, bits, seed=11, n_samples=3)  # empty tensor: zeros, nothing launched on the area


def test_a_tensor_beyond_the_scratch_area_is_refused_before_any_launch(gact):
    tiles = gact.GACT_NOALLOC_SCRATCH_BYTES // 8
    x = torch.zeros(4096, dtype=torch.float32, device="cuda")
    packed, gmin, gscale = gact.alloc_compressed(4096, 256, 2, x.device)
    fp = torch.zeros(9, dtype=torch.float64, device="cuda")
    # sizes are checked on the host before anything is enqueued, so the small buffers are never touched
    rc = gact.lib.gact_compress_footprint_noalloc(x.data_ptr(), gact.GACT_F32, tiles * 2048 + 1, 256, 2, 0,
                                                  packed.data_ptr(), gmin.data_ptr(), gscale.data_ptr(), 8,
                                                  fp.data_ptr(), None)
    assert rc == gact.GACT_E_SCRATCH
    assert "scratch" in gact.error_string(rc)
    with pytest.raises(gact.GactError):
        gact.gact_compress_footprint_noalloc(x, 48, 2, 0, 8, packed, gmin, gscale, fp)     # bad group size
