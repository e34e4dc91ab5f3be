"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the
same seeded inputs.  Packed codes, group minima and steps must be bit-exact;
dequantised values within 1e-6 relative (fp32) / one bf16 ulp -- in practice
they are compared for equality first and the tolerance is the stated bar.
Quantizer: arXiv 2206.11357 App. A.4, per group (Sec. 5)."""
import os
import sys

import numpy as np
import pytest
import torch

import oracle
import synthetic_inputs as syn

pytestmark = pytest.mark.gpu

CANARY = 0xA5
PAD = 256        # guard bytes after every output buffer


def to_device(x_np):
    """numpy float32 / uint16(bf16 bits) -> device tensor of the matching dtype"""
    if x_np.dtype == np.uint16:
        return torch.from_numpy(x_np.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(x_np).cuda()


def to_host(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def guarded(nbytes, dtype):
    """A buffer of nbytes followed by PAD canary bytes; returns (view, whole)."""
    whole = torch.full((nbytes + PAD,), CANARY, dtype=torch.uint8, device="cuda")
    return whole[:nbytes].view(dtype), whole


def canary_intact(whole, nbytes):
    return bool((whole[nbytes:] == CANARY).all().item())


def run_case(gact, x_np, G, bits, seed, check_y=True):
    """Compress + decompress on the GPU with guarded buffers; compare to oracle."""
    n = x_np.size
    x = to_device(x_np)
    x_before = x.clone()
    pb = gact.gact_packed_bytes(n, bits)
    ng = gact.gact_num_groups(n, G)
    packed, packed_w = guarded(pb, torch.uint8)
    gmin, gmin_w = guarded(ng * 4, torch.float32)
    gscale, gscale_w = guarded(ng * 4, torch.float32)
    gact.gact_compress(x, G, bits, seed, packed, gmin, gscale)
    y, y_w = guarded(n * x.element_size(), x.dtype)
    gact.gact_decompress(packed, gmin, gscale, n, G, bits, y=y)
    torch.cuda.synchronize()

    p_ref, mn_ref, sc_ref = oracle.compress(x_np, G, bits, seed)
    assert torch.equal(x, x_before), "compress modified its input"
    assert canary_intact(packed_w, pb) and canary_intact(gmin_w, ng * 4)
    assert canary_intact(gscale_w, ng * 4) and canary_intact(y_w, n * x.element_size())
    mn, sc, p = to_host(gmin), to_host(gscale), to_host(packed)
    assert np.array_equal(mn.view(np.uint32), mn_ref.view(np.uint32)), "gmin differs"
    assert np.array_equal(sc.view(np.uint32), sc_ref.view(np.uint32)), "gscale differs"
    if not np.array_equal(p, p_ref):
        bad = np.flatnonzero(p != p_ref)
        raise AssertionError("packed differs at %d bytes, first %s" % (bad.size, bad[:8]))
    if check_y:
        dt = oracle.BF16 if x_np.dtype == np.uint16 else oracle.F32
        y_ref = oracle.decompress(p_ref, mn_ref, sc_ref, n, G, bits, dt)
        y_h = to_host(y)
        if dt == oracle.F32:
            # bar: 1e-6 relative; the two sides run the same two roundings
            assert np.allclose(y_h, y_ref, rtol=1e-6, atol=0)
            assert np.array_equal(y_h.view(np.uint32), y_ref.view(np.uint32))
        else:
            # bar: one bf16 ulp
            assert np.all(np.abs(y_h.astype(np.int32) - y_ref.astype(np.int32)) <= 1)
            assert np.array_equal(y_h, y_ref)
    return p, mn, sc


# ------------------------------------------------------------------ config 1
def test_config1_single_tensor(gact):
    c = syn.config1()
    run_case(gact, c["x"], c["group_size"], c["bits"], c["seed"])


# ------------------------------------------------- sizes, tiles, ragged tails
@pytest.mark.parametrize("dtype", ("f32", "bf16"))
@pytest.mark.parametrize("bits", (1, 2, 4, 8))
@pytest.mark.parametrize("G", (32, 128, 256, 1024))
def test_tiles_and_ragged_tails(gact, dtype, bits, G):
    # several wavefront tiles (2048 elements) and blocks (8192), ends inside a
    # tile, inside a group, inside a 16-byte load and inside a Philox block
    for n in (1, 5, 31, 33, 2048, 2049, 8192 + 7, 5 * 8192 + 3 * 256 + 129, 40000 - 1):
        x = syn.draw_numpy(syn.OUTLIER, n, 100 + n % 97)
        if dtype == "bf16":
            x = syn.f32_to_bf16_bits(x)
        run_case(gact, x, G, bits, seed=n + bits)


@pytest.mark.parametrize("dtype", ("f32", "bf16"))
@pytest.mark.parametrize("G", (64, 96, 160, 352, 512, 736, 992))
def test_other_group_sizes(gact, dtype, G):
    for n, bits in ((G * 70 + 13, 2), (G * 21, 1), (G * 64, 4), (3 * G - 1, 8), (2016 * 3, 1)):
        x = syn.draw_numpy(syn.NORMAL, n, G + bits)
        if dtype == "bf16":
            x = syn.f32_to_bf16_bits(x)
        run_case(gact, x, G, bits, seed=G)


def test_value_laws_of_the_workloads(gact):
    # half-zero ReLU outputs, GELU outputs, softmax rows (values in [0,1], skewed)
    for law, row, dtype, G, bits in ((syn.RELU, 0, "f32", 256, 2), (syn.RELU, 0, "f32", 256, 4),
                                     (syn.SOFTMAX, 512, "bf16", 256, 4), (syn.GELU, 0, "bf16", 128, 2),
                                     (syn.SOFTMAX, 197, "bf16", 128, 8), (syn.NORMAL, 0, "bf16", 128, 1)):
        n = 197 * 512 * 3 if law == syn.SOFTMAX else 100000
        x = syn.draw_numpy(law, n, 7, row)
        if dtype == "bf16":
            x = syn.f32_to_bf16_bits(x)
        run_case(gact, x, G, bits, seed=3)


# ------------------------------------------------------------ degenerate cases
@pytest.mark.parametrize("bits", (1, 2, 4, 8))
def test_constant_zero_tiny_range_and_signed_zero_groups(gact, bits):
    G = 64
    x = syn.draw_numpy(syn.NORMAL, 40 * G, 1)
    x[0:G] = 3.25                       # constant
    x[G:2 * G] = 0.0
    x[G + 5] = -0.0                     # signed zeros only
    x[2 * G:3 * G] = 1e-30
    x[2 * G + 1] = np.float32(1e-30) + np.float32(2.0**-110)      # range below 2^-100
    x[3 * G:4 * G] = np.abs(x[3 * G:4 * G]); x[3 * G + 9] = -0.0   # minimum is -0
    x[4 * G:5 * G] = np.float32(2.0**-100) * np.arange(G)          # range just above the threshold
    x[5 * G:6 * G] = 1e30 * x[5 * G:6 * G]                         # large magnitudes
    x[6 * G:7 * G] = -5.0; x[6 * G + 63] = 5.0                     # two-valued
    p, mn, sc = run_case(gact, x, G, bits, seed=9)
    assert sc[0] == 0 and sc[1] == 0 and sc[2] == 0
    assert not np.signbit(mn[1]) and not np.signbit(mn[3])


@pytest.mark.parametrize("bits", (1, 2, 4, 8))
def test_on_grid_inputs_round_trip_exactly(gact, bits):
    B = 2 ** bits - 1
    G = 256
    rng = np.random.default_rng(bits)
    j = rng.integers(0, B + 1, size=16 * G)
    j[::G] = 0
    j[1::G] = B
    x = (np.float32(-4.0) + j * np.float32(0.125)).astype(np.float32)
    xd = torch.from_numpy(x).cuda()
    for seed in (0, 1, 2**40 + 17):
        packed, gmin, gscale = gact.gact_compress(xd, G, bits, seed)
        y = gact.gact_decompress(packed, gmin, gscale, x.size, G, bits)
        assert torch.equal(y, xd)
    run_case(gact, x, G, bits, seed=5)


def test_top_code_is_clamped_under_eight_bits(gact):
    # many groups whose (max-min)*fl(255/(max-min)) overshoots 255 by an ulp
    x = syn.draw_numpy(syn.NORMAL, 32 * 20000, 2)
    p, mn, sc = run_case(gact, x, 32, 8, seed=11, check_y=False)
    top = x.reshape(-1, 32).argmax(1) + np.arange(20000) * 32
    assert np.all(p[top] >= 254)


def test_non_finite_inputs_do_not_write_out_of_bounds(gact):
    x = syn.draw_numpy(syn.NORMAL, 5000, 3)
    x[17] = np.nan; x[300] = np.inf; x[2100] = -np.inf; x[4999] = np.nan
    xd = torch.from_numpy(x).cuda()
    n, G, bits = x.size, 128, 4
    pb, ng = gact.gact_packed_bytes(n, bits), gact.gact_num_groups(n, G)
    packed, pw = guarded(pb, torch.uint8)
    gmin, mw = guarded(ng * 4, torch.float32)
    gscale, sw = guarded(ng * 4, torch.float32)
    y, yw = guarded(n * 4, torch.float32)
    gact.gact_compress(xd, G, bits, 1, packed, gmin, gscale)
    gact.gact_decompress(packed, gmin, gscale, n, G, bits, y=y)
    torch.cuda.synchronize()
    assert canary_intact(pw, pb) and canary_intact(mw, ng * 4) and canary_intact(sw, ng * 4)
    assert canary_intact(yw, n * 4)


# ------------------------------------------------------- seeds and large index
def test_seed_words_and_replay(gact):
    x = syn.draw_numpy(syn.NORMAL, 10000, 4)
    for seed in (0, 1, 0xFFFFFFFF, 1 << 32, 0x0123456789ABCDEF, 2**64 - 1):
        run_case(gact, x, 256, 2, seed, check_y=False)
    xd = torch.from_numpy(x).cuda()
    a = gact.gact_compress(xd, 256, 2, 77)
    b = gact.gact_compress(xd, 256, 2, 77)
    c = gact.gact_compress(xd, 256, 2, 78)
    assert torch.equal(a[0], b[0]) and not torch.equal(a[0], c[0])
    assert torch.equal(a[1], c[1]) and torch.equal(a[2], c[2])


# ------------------------------------------------------------------ multi-tensor
def multi_case(gact, specs, G):
    """specs: list of (x_np, bits, seed).  Runs both multi calls with guarded
    buffers and compares every tensor with the oracle and the single calls."""
    L = len(specs)
    xs = [to_device(x) if x.size else torch.empty(0, device="cuda", dtype=torch.float32 if x.dtype == np.float32 else torch.bfloat16) for x, _, _ in specs]
    ns = [x.size for x, _, _ in specs]
    bits = [b for _, b, _ in specs]
    seeds = [s for _, _, s in specs]
    dts = [t.dtype for t in xs]
    bufs = []
    for l in range(L):
        pb, ng = gact.gact_packed_bytes(ns[l], bits[l]), gact.gact_num_groups(ns[l], G)
        bufs.append((guarded(pb, torch.uint8), guarded(ng * 4, torch.float32),
                     guarded(ng * 4, torch.float32), guarded(ns[l] * xs[l].element_size(), dts[l]),
                     pb, ng))
    descs = gact.make_descs(xs, [b[0][0] for b in bufs], [b[1][0] for b in bufs],
                            [b[2][0] for b in bufs], [b[3][0] for b in bufs], ns, bits, seeds, dts)
    ws = torch.empty(gact.gact_multi_workspace_bytes(L), dtype=torch.uint8, device="cuda")
    gact.gact_compress_multi(descs, L, G, ws)
    gact.gact_decompress_multi(descs, L, G, ws)
    torch.cuda.synchronize()
    for l, (x_np, b, s) in enumerate(specs):
        (p, pw), (mn, mw), (sc, sw), (y, yw), pb, ng = bufs[l]
        assert canary_intact(pw, pb) and canary_intact(mw, ng * 4) and canary_intact(sw, ng * 4)
        assert canary_intact(yw, ns[l] * xs[l].element_size())
        if ns[l] == 0:
            continue
        p_ref, mn_ref, sc_ref = oracle.compress(x_np, G, b, s)
        dt = oracle.BF16 if x_np.dtype == np.uint16 else oracle.F32
        y_ref = oracle.decompress(p_ref, mn_ref, sc_ref, ns[l], G, b, dt)
        assert np.array_equal(to_host(p), p_ref), l
        assert np.array_equal(to_host(mn).view(np.uint32), mn_ref.view(np.uint32)), l
        assert np.array_equal(to_host(sc).view(np.uint32), sc_ref.view(np.uint32)), l
        yh = to_host(y)
        assert np.array_equal(yh.view(np.uint32) if dt == oracle.F32 else yh,
                              y_ref.view(np.uint32) if dt == oracle.F32 else y_ref), l
        # single-tensor call gives the same bytes (launch-shape independence)
        p1, mn1, sc1 = gact.gact_compress(xs[l], G, b, s)
        assert torch.equal(p1, p) and torch.equal(mn1, mn) and torch.equal(sc1, sc)


@pytest.mark.parametrize("G", (128, 256, 96))
def test_multi_tensor_mixed_set(gact, G):
    rng = np.random.default_rng(G)
    specs = []
    sizes = [0, 1, 100, 2048, 8192, 8193, 30000, 128 * 1000, 128 * 1024, 0, 70001, 197 * 197 * 4]
    for k, n in enumerate(sizes):
        x = syn.draw_numpy(syn.NORMAL if k % 2 else syn.RELU, n, 50 + k) if n else np.empty(0, np.float32)
        if k % 3 == 0:
            x = syn.f32_to_bf16_bits(x) if n else np.empty(0, np.uint16)
        specs.append((x, int(rng.choice([1, 2, 4, 8])), int(rng.integers(0, 2**63))))
    multi_case(gact, specs, G)


def test_multi_tensor_many_small(gact):
    rng = np.random.default_rng(0)
    specs = [(syn.f32_to_bf16_bits(syn.draw_numpy(syn.NORMAL, int(rng.integers(1, 6000)), k)),
              int(rng.choice([1, 2, 4, 8])), k) for k in range(400)]
    multi_case(gact, specs, 128)


# ------------------------------------------------------ allocator feeds multi
def test_allocator_bits_drive_a_multi_launch(gact):
    L = 24
    c = syn.lognormal_sensitivities(L, 2999)
    ns = [int(v) for v in np.random.default_rng(1).integers(1, 40, L) * 256]
    bits = gact.gact_allocate_bits(c, ns, 2.0)
    assert np.array_equal(bits, oracle.allocate_bits(c, ns, 2.0))
    specs = [(syn.draw_numpy(syn.RELU, ns[l], 2000 + l), int(bits[l]), l) for l in range(L)]
    multi_case(gact, specs, 256)


def test_uncompressed_level_is_skipped_by_the_multi_calls(gact):
    """bits = 32 in a descriptor: the allocator left the tensor at full
    precision; neither call touches its buffers."""
    L, G = 10, 256
    c = syn.lognormal_sensitivities(L, 77)
    c[3] = 1e9                                   # far more sensitive than the rest
    ns = [int(v) * 256 for v in np.random.default_rng(2).integers(4, 60, L)]
    avg = float((32 * ns[3] + 4 * (sum(ns) - ns[3])) / sum(ns))   # one tensor at 32, the rest at 4
    bits = gact.gact_allocate_bits_levels(c, ns, avg, (1, 2, 4, 8, 32))
    assert np.array_equal(bits, oracle.allocate_bits_levels(c, ns, avg, (1, 2, 4, 8, 32)))
    assert bits[3] == 32 and np.all(np.delete(bits, 3) < 32)
    x_np = [syn.draw_numpy(syn.NORMAL, ns[l], 300 + l) for l in range(L)]
    xs = [torch.from_numpy(x).cuda() for x in x_np]
    bufs = [gact.alloc_compressed(ns[l], G, 8, "cuda") for l in range(L)]
    for p, mn, sc in bufs:
        p.fill_(CANARY); mn.fill_(-7.0); sc.fill_(-7.0)
    ys = [torch.full_like(x, -3.0) for x in xs]
    descs = gact.make_descs(xs, [b[0] for b in bufs], [b[1] for b in bufs], [b[2] for b in bufs], ys,
                            ns, bits, list(range(L)), [x.dtype for x in xs])
    ws = torch.empty(gact.gact_multi_workspace_bytes(L), dtype=torch.uint8, device="cuda")
    gact.gact_compress_multi(descs, L, G, ws)
    gact.gact_decompress_multi(descs, L, G, ws)
    torch.cuda.synchronize()
    assert bool((bufs[3][0] == CANARY).all()) and bool((bufs[3][1] == -7.0).all())
    assert bool((ys[3] == -3.0).all())
    for l in range(L):
        if l == 3:
            continue
        p_ref, mn_ref, sc_ref = oracle.compress(x_np[l], G, int(bits[l]), l)
        nb = p_ref.size
        assert np.array_equal(bufs[l][0][:nb].cpu().numpy(), p_ref)
        assert np.array_equal(ys[l].cpu().numpy(), oracle.decompress(p_ref, mn_ref, sc_ref, ns[l], G, int(bits[l])))


# ------------------------------------------------------------- frozen digests
def test_hip_path_reproduces_the_oracle_s_frozen_digests(gact):
    """The digests in tests/golden/oracle_digests.txt were written from the CPU
    oracle alone; the HIP path must hash to the same values on the same inputs."""
    import hashlib
    here = os.path.dirname(os.path.abspath(__file__))
    sys.path.insert(0, os.path.join(here, "golden"))
    import make_golden
    with open(os.path.join(here, "golden", "oracle_digests.txt")) as f:
        stored = {ln.split()[0]: dict(kv.split("=") for kv in ln.split()[1:])
                  for ln in f if not ln.startswith("#")}
    sha = lambda a: hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()
    for name, x, G, b, seed in make_golden.codec_cases():
        want = stored[name]
        assert sha(x) == want["input"], name
        xd = to_device(x)
        p, mn, sc = gact.gact_compress(xd, G, b, seed)
        y = gact.gact_decompress(p, mn, sc, x.size, G, b, dtype=xd.dtype)
        assert sha(to_host(p)) == want["packed"], name
        assert sha(to_host(mn)) == want["gmin"] and sha(to_host(sc)) == want["gscale"], name
        assert sha(to_host(y)) == want["dequantised"], name


# ------------------------------------------------------------------ HIP graphs
def test_multi_launches_replay_correctly_from_a_captured_graph(gact):
    """Up to 64 tensors the launch table travels in the kernel arguments, so a
    compress + decompress pair is two kernel nodes and nothing else.  The graph
    is replayed several times on changed inputs, with eager work and
    synchronisation in between, and every replay is checked against the oracle."""
    G, L = 256, 6
    ns = [5000, 8192, 70001, 1, 33000, 2048 * 9]
    bits = [2, 4, 1, 8, 2, 4]
    seeds = [11, 12, 13, 14, 15, 16]
    dts = [torch.float32, torch.bfloat16, torch.float32, torch.float32, torch.bfloat16, torch.float32]
    xs = [torch.zeros(n, device="cuda", dtype=dt) for n, dt in zip(ns, dts)]
    bufs = [gact.alloc_compressed(n, G, b, "cuda") for n, b in zip(ns, bits)]
    ys = [torch.empty_like(x) for x in xs]
    descs = gact.make_descs(xs, [b[0] for b in bufs], [b[1] for b in bufs], [b[2] for b in bufs], ys,
                            ns, bits, seeds, dts)
    ws = torch.empty(gact.gact_multi_workspace_bytes(L), dtype=torch.uint8, device="cuda")

    def fill(round_):
        host = []
        for l in range(L):
            x = syn.draw_numpy(syn.NORMAL if l % 2 else syn.RELU, ns[l], 900 + 10 * round_ + l)
            if dts[l] == torch.bfloat16:
                x = syn.f32_to_bf16_bits(x)
            xs[l].copy_(to_device(x))
            host.append(x)
        return host

    side = torch.cuda.Stream()                       # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                    # warm-up outside the capture
        fill(0)
        gact.gact_compress_multi(descs, L, G, ws)
        gact.gact_decompress_multi(descs, L, G, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gact.gact_compress_multi(descs, L, G, ws)
        gact.gact_decompress_multi(descs, L, G, ws)
    for round_ in (1, 2, 3):
        host = fill(round_)                          # eager copies between the replays
        for b in bufs:
            b[0].fill_(CANARY)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(L):
            p_ref, mn_ref, sc_ref = oracle.compress(host[l], G, bits[l], seeds[l])
            dt = oracle.BF16 if host[l].dtype == np.uint16 else oracle.F32
            y_ref = oracle.decompress(p_ref, mn_ref, sc_ref, ns[l], G, bits[l], dt)
            assert np.array_equal(to_host(bufs[l][0])[:p_ref.size], p_ref), (round_, l)
            assert np.array_equal(to_host(bufs[l][1]).view(np.uint32), mn_ref.view(np.uint32)), (round_, l)
            assert np.array_equal(to_host(bufs[l][2]).view(np.uint32), sc_ref.view(np.uint32)), (round_, l)
            yh = to_host(ys[l])
            assert np.array_equal(yh.view(np.uint32) if dt == oracle.F32 else yh,
                                  y_ref.view(np.uint32) if dt == oracle.F32 else y_ref), (round_, l)


def test_a_table_upload_is_refused_on_a_capturing_stream(gact):
    """More than 64 tensors need their table uploaded from host memory, which a
    graph replay could not repeat: under capture the call enqueues nothing and
    says so; the same call works once the capture has ended."""
    G, L = 128, 70
    xs = [torch.from_numpy(syn.draw_numpy(syn.NORMAL, 4096, 700 + l)).cuda() for l in range(L)]
    bufs = [gact.alloc_compressed(4096, G, 4, "cuda") for _ in range(L)]
    ys = [torch.empty_like(x) for x in xs]
    descs = gact.make_descs(xs, [b[0] for b in bufs], [b[1] for b in bufs], [b[2] for b in bufs], ys,
                            [4096] * L, [4] * L, list(range(L)), [torch.float32] * L)
    ws = torch.empty(gact.gact_multi_workspace_bytes(L), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    codes = []
    with torch.cuda.graph(graph):
        for call in (gact.gact_compress_multi, gact.gact_decompress_multi):
            try:
                call(descs, L, G, ws)
                codes.append(0)
            except gact.GactError as e:
                codes.append(e.code)
    assert codes == [gact.GACT_E_CAPTURE, gact.GACT_E_CAPTURE]
    gact.gact_compress_multi(descs, L, G, ws)
    gact.gact_decompress_multi(descs, L, G, ws)
    torch.cuda.synchronize()
    p_ref, mn_ref, sc_ref = oracle.compress(xs[69].cpu().numpy(), G, 4, 69)
    assert np.array_equal(to_host(bufs[69][0]), p_ref)
    assert np.array_equal(ys[69].cpu().numpy(), oracle.decompress(p_ref, mn_ref, sc_ref, 4096, G, 4))


def test_calls_on_two_streams_do_not_interfere(gact):
    """The library keeps no state between calls: launches enqueued on two
    streams at the same time (each with its own buffers and workspace) give the
    oracle's bytes."""
    G = 256
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]          # default priority
    jobs = []
    for k, s in enumerate(streams):
        x_np = [syn.draw_numpy(syn.NORMAL, 300000 + 4097 * k, 40 + k), syn.draw_numpy(syn.RELU, 8192 * 30, 50 + k)]
        bits = [2 + 2 * k, 1 + 7 * k]
        with torch.cuda.stream(s):
            xs = [to_device(x) for x in x_np]
            bufs = [gact.alloc_compressed(x.size, G, b, "cuda") for x, b in zip(x_np, bits)]
            ys = [torch.empty_like(x) for x in xs]
            descs = gact.make_descs(xs, [b[0] for b in bufs], [b[1] for b in bufs], [b[2] for b in bufs], ys,
                                    [x.size for x in x_np], bits, [k, k + 10], [torch.float32] * 2)
            ws = torch.empty(gact.gact_multi_workspace_bytes(2), dtype=torch.uint8, device="cuda")
        jobs.append((s, x_np, bits, xs, bufs, ys, descs, ws))
    for _ in range(5):                                             # interleave the launches
        for s, x_np, bits, xs, bufs, ys, descs, ws in jobs:
            with torch.cuda.stream(s):
                gact.gact_compress_multi(descs, 2, G, ws)
                gact.gact_decompress_multi(descs, 2, G, ws)
    torch.cuda.synchronize()
    for k, (s, x_np, bits, xs, bufs, ys, descs, ws) in enumerate(jobs):
        for l in range(2):
            p_ref, mn_ref, sc_ref = oracle.compress(x_np[l], G, bits[l], k + 10 * l)
            assert np.array_equal(to_host(bufs[l][0]), p_ref), (k, l)
            assert np.array_equal(to_host(ys[l]), oracle.decompress(p_ref, mn_ref, sc_ref, x_np[l].size, G, bits[l])), (k, l)


# ---------------------------------------------------------------------- shards
@pytest.mark.parametrize("dtype,G,bits", [("f32", 256, 2), ("bf16", 128, 4), ("f32", 96, 8), ("bf16", 1024, 1)])
def test_shards_with_an_index_base_concatenate_to_the_whole(gact, dtype, G, bits):
    """A tensor cut at multiples of the group size and compressed shard by shard,
    each with the tensor's seed and its own offset in the noise stream, gives
    the bytes of the whole tensor: what one GPU of a sharded tensor would do.
    Each shard also equals the oracle's result for that slice."""
    n, seed = 50 * G * 37 + 77, 2**40 + 9
    x = syn.draw_numpy(syn.NORMAL, n, 61)
    if dtype == "bf16":
        x = syn.f32_to_bf16_bits(x)
    cuts = [0, 7 * G, 7 * G + 32 * G, 900 * G, n]                       # four shards, the last one ragged
    assert bits * G % 128 == 0 or all((c * bits) % 128 == 0 for c in cuts[:-1])   # shard strings end on 16-byte units
    xd = to_device(x)
    whole = gact.gact_compress(xd, G, bits, seed)
    xs, bufs, ns, bases = [], [], [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        xs.append(xd[a:b].clone())                                      # own 16-byte aligned buffer
        bufs.append(gact.alloc_compressed(b - a, G, bits, "cuda"))
        ns.append(b - a); bases.append(a)
    L = len(ns)
    descs = gact.make_descs(xs, [b[0] for b in bufs], [b[1] for b in bufs], [b[2] for b in bufs],
                            [None] * L, ns, [bits] * L, [seed] * L, [xd.dtype] * L, index_bases=bases)
    ws = torch.empty(gact.gact_multi_workspace_bytes(L), dtype=torch.uint8, device="cuda")
    gact.gact_compress_multi(descs, L, G, ws)
    torch.cuda.synchronize()
    for k, (a, b) in enumerate(zip(cuts[:-1], cuts[1:])):
        p_ref, mn_ref, sc_ref = oracle.compress_slice(x[a:b], G, bits, seed, a)
        assert np.array_equal(to_host(bufs[k][0]), p_ref), k
        assert np.array_equal(to_host(bufs[k][1]).view(np.uint32), mn_ref.view(np.uint32)), k
        assert np.array_equal(to_host(bufs[k][2]).view(np.uint32), sc_ref.view(np.uint32)), k
    pb = [gact.gact_packed_bytes(m, bits) for m in ns]
    exact = [m * bits // 8 for m in ns]                                  # bytes before the 16-byte padding
    cat = torch.cat([bufs[k][0][:exact[k]] for k in range(L - 1)] + [bufs[L - 1][0]])
    assert torch.equal(cat, whole[0])
    assert torch.equal(torch.cat([b[1] for b in bufs]), whole[1])
    assert torch.equal(torch.cat([b[2] for b in bufs]), whole[2])
    # a shard compressed without its offset draws other noise
    other = gact.gact_compress(xs[1], G, bits, seed)
    assert not torch.equal(other[0], bufs[1][0])


def test_index_base_beyond_32_bit_block_numbers(gact):
    """Offsets whose Philox block number needs more than 32 bits reach the
    counter's high word; checked against the oracle's slice at the same offset."""
    G, bits, seed, n = 128, 4, 77, 5000
    x = syn.draw_numpy(syn.RELU, n, 62)
    xd = to_device(x)
    for base in (2**35, 2**43 + 2**35 + 128 * 3, (2**48 - 1) * 8 // 128 * 128):
        p, mn, sc = gact.alloc_compressed(n, G, bits, "cuda")
        descs = gact.make_descs([xd], [p], [mn], [sc], [None], [n], [bits], [seed], [xd.dtype], index_bases=[base])
        ws = torch.empty(gact.gact_multi_workspace_bytes(1), dtype=torch.uint8, device="cuda")
        gact.gact_compress_multi(descs, 1, G, ws)
        p_ref, mn_ref, sc_ref = oracle.compress_slice(x, G, bits, seed, base)
        assert np.array_equal(to_host(p), p_ref), base
        assert np.array_equal(to_host(mn).view(np.uint32), mn_ref.view(np.uint32)), base


def test_multi_tensor_three_thousand_tiny_tensors(gact):
    """A long table (uploaded to the workspace, 12 search steps per block) of
    tensors that are mostly smaller than one tile."""
    rng = np.random.default_rng(5)
    specs = []
    for k in range(3000):
        n = int(rng.integers(1, 700))
        x = syn.draw_numpy(syn.NORMAL, n, 9000 + k)
        if k % 2:
            x = syn.f32_to_bf16_bits(x)
        specs.append((x, int(rng.choice([1, 2, 4, 8])), k))
    multi_case(gact, specs, 64)


def test_prepared_calls_give_the_same_bytes_as_the_plain_calls(gact):
    """A call marshalled once and issued repeatedly (PreparedCall) is the same C call: same bytes, on the
    default stream and on a side stream."""
    n, G, bits, seed = 3 * 8192 + 321, 128, 4, 77
    x_np = syn.f32_to_bf16_bits(syn.draw_numpy(syn.NORMAL, n, 31))
    x = to_device(x_np)
    ref = gact.gact_compress(x, G, bits, seed)
    y_ref = gact.gact_decompress(*ref, n, G, bits, dtype=x.dtype)
    bufs = gact.alloc_compressed(n, G, bits, x.device)
    y = torch.empty_like(x)
    comp = gact.prepare_compress(x, G, bits, seed, *bufs)
    dec = gact.prepare_decompress(*bufs, n, G, bits, y)
    side = torch.cuda.Stream()
    for stream in (torch.cuda.current_stream(), side):
        for t in bufs:
            t.view(torch.uint8).fill_(0)
        y.view(torch.int16).fill_(0)
        torch.cuda.synchronize()
        comp(stream.cuda_stream)
        dec(stream.cuda_stream)
        stream.synchronize()
        for got, want in zip(bufs, ref):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16))
    p_ref, mn_ref, sc_ref = oracle.compress(x_np, G, bits, seed)
    assert np.array_equal(to_host(bufs[0]), p_ref)


def test_bounded_copy_moves_every_byte_both_ways_and_refuses_pageable_memory(gact):
    """The swap copy of Sec. 5.3: device to pinned host memory and back, sizes with and without a
    16-byte tail, few and many workgroups; ordinary host memory is refused before any launch."""
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev).manual_seed(5)
    for nbytes, wg in ((16, 1), (4096 + 7, 3), (1 << 20, 16), ((5 << 20) + 13, 16), ((3 << 20) + 16, 1024)):
        src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=dev, generator=g)
        host = torch.zeros(nbytes + 32, dtype=torch.uint8, pin_memory=True)
        gact.gact_copy_bounded(host[:nbytes], src, wg)
        torch.cuda.synchronize()
        assert torch.equal(host[:nbytes], src.cpu()) and int(host[nbytes:].sum()) == 0
        back = torch.zeros(nbytes + 32, dtype=torch.uint8, device=dev)
        gact.gact_copy_bounded(back[:nbytes], host[:nbytes], wg)
        torch.cuda.synchronize()
        assert torch.equal(back[:nbytes], src) and int(back[nbytes:].sum()) == 0
    with pytest.raises(gact.GactError):
        gact.gact_copy_bounded(torch.empty(1024, dtype=torch.uint8), src[:1024], 16)
    with pytest.raises(ValueError):
        gact.gact_copy_bounded(host[:64], src[:128], 16)
    torch.cuda.synchronize()
