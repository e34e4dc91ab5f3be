#!/usr/bin/env python3
"""Throughput of the GACT compress + decompress hot path on one MI355X.

A step = one pass of the whole path over one synthetic activation set, inputs
already resident in HBM: host bit allocation (Eq. (ilp) of arXiv 2206.11357),
one multi-tensor compress launch, one multi-tensor decompress launch.

Prints ONE JSON line.  `value` is uncompressed GB/s averaged over the two
directions: (bytes read by compress + bytes written by decompress) / time.
`roofline` prices the dominant kernel (compress) in algorithmic bytes
(sizeof(T) + bits/8 + 8/G per element) against the 8 TB/s HBM3E peak, with its
launch duration measured by events on the launch stream inside the timed
steps.  `cpu_baseline` is the CPU oracle timed on a bounded sample of the same
tensors on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E, published

WORKLOADS = {
    # name: (set builder, group size, average bits, sensitivity seed, description)
    "resnet50_b64": ("resnet50_set", 256, 2.0, 2999,
                     "53 conv outputs of a ResNet-50-shaped net, batch 64, fp32, G=256, allocator avg 2 bits"),
    "bert_large_b32": ("bert_large_set", 256, 4.0, 3999,
                       "96 saved tensors of a BERT-large-shaped encoder, batch 32 x seq 512, bf16, G=256, allocator avg 4 bits"),
    "gcn_arxiv": ("gcn_set", 256, 2.0, 4999,
                  "3 GCN activations 169343 x 256, fp32, G=256, 2 bits"),
    "vit_large_b128": ("vit_large_set", 128, 3.0, 5999,
                       "400 saved tensors of a ViT-L/16-shaped model, batch 128, bf16, G=128, allocator avg 3 bits"),
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="resnet50_b64",
                    choices=sorted(WORKLOADS) + ["grad_sensitivity"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-elems", type=int, default=800_000_000)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the workload, launch a plain elementwise kernel that reads "
                         "1 GiB and writes 1 GiB five times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no cross-GPU step and this build runs on "
              "single-GPU boxes; run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2206_11357_amd as gact
    import synthetic_inputs as syn

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "kernel": "torch.add(src, 1.0, out=dst)",
                          "read_bytes_per_launch": src.numel() * 4,
                          "write_bytes_per_launch": dst.numel() * 4, "launches": 5}))
        return 0

    if args.workload == "grad_sensitivity":
        return bench_grad_sensitivity(args, gact, torch, np, dev)

    builder, G, avg_bits, sens_seed, desc = WORKLOADS[args.workload]
    specs = getattr(syn, builder)()
    L = len(specs)
    numel = np.array([s.numel for s in specs], dtype=np.int64)
    sens = syn.lognormal_sensitivities(L, sens_seed)
    if args.workload == "gcn_arxiv":
        sens[:] = 1.0                       # fixed 2 bits everywhere
    torch_dt = {"f32": torch.float32, "bf16": torch.bfloat16}
    esize = {"f32": 4, "bf16": 2}

    # inputs resident in HBM before anything is timed
    xs = [syn.draw_torch(s, dev) for s in specs]
    bits = gact.gact_allocate_bits(sens, numel, avg_bits)
    # buffers sized for the widest code so that any allocation result fits
    packed, gmin, gscale, ys = [], [], [], []
    for s, x in zip(specs, xs):
        p, mn, sc = gact.alloc_compressed(s.numel, G, 8, dev)
        packed.append(p); gmin.append(mn); gscale.append(sc)
        ys.append(torch.empty_like(x))
    ws = torch.empty(gact.gact_multi_workspace_bytes(L), dtype=torch.uint8, device=dev)
    seeds = [s.seed for s in specs]
    dts = [torch_dt[s.dtype] for s in specs]
    torch.cuda.synchronize()

    ev = lambda: torch.cuda.Event(enable_timing=True)
    c_ms, d_ms = [], []

    def step(record: bool):
        b = gact.gact_allocate_bits(sens, numel, avg_bits)
        descs = gact.make_descs(xs, packed, gmin, gscale, ys, numel, b, seeds, dts)
        if record:
            e0, e1, e2 = ev(), ev(), ev()
            e0.record()
        gact.gact_compress_multi(descs, L, G, ws)
        if record:
            e1.record()
        gact.gact_decompress_multi(descs, L, G, ws)
        if record:
            e2.record()
            return e0, e1, e2
        return None

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks = [step(True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for e0, e1, e2 in marks:
        c_ms.append(e0.elapsed_time(e1))
        d_ms.append(e1.elapsed_time(e2))

    ms_per_step = wall * 1e3 / args.steps
    n_total = int(numel.sum())
    in_bytes = int(sum(int(n) * esize[s.dtype] for n, s in zip(numel, specs)))
    packed_bytes = int(sum(gact.gact_packed_bytes(int(n), int(b)) for n, b in zip(numel, bits)))
    meta_bytes = int(sum(8 * gact.gact_num_groups(int(n), G) for n in numel))
    alg_bytes = in_bytes + packed_bytes + meta_bytes          # per direction
    c_avg, d_avg = float(np.mean(c_ms)), float(np.mean(d_ms))
    value = 2.0 * in_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = alg_bytes / (c_avg * 1e-3) / 1e9

    # HBM bytes per compress launch from the committed counter summary (null if none)
    traffic = None
    try:
        import re
        for name in sorted(os.listdir(os.path.join(ROOT, "profiles"))):
            text = open(os.path.join(ROOT, "profiles", name)).read()
            m = re.search(r"traffic_compress_bytes_per_launch\[%s\]\s*=\s*(\d+)" % re.escape(args.workload), text)
            if m:
                traffic = int(m.group(1))
    except OSError:
        traffic = None

    out = {
        "metric": "compress+decompress GB/s (input bytes) and % of HBM peak, 1xMI355X",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": args.workload, "description": desc, "tensors": L, "elements": n_total,
            "group_size": G, "avg_bits": avg_bits,
            "bits_histogram": {str(k): int((bits == k).sum()) for k in (1, 2, 4, 8)},
            "input_bytes": in_bytes, "algorithmic_bytes_per_direction": alg_bytes,
            "launch": "one multi-tensor launch per direction",
        },
        "compress": {"ms": round(c_avg, 4), "input_GBps": round(in_bytes / c_avg / 1e6, 1),
                     "elements_per_s": round(n_total / c_avg * 1e3, 0),
                     "pct_hbm_peak": round(100 * alg_bytes / c_avg / 1e6 / HBM_PEAK_GBPS, 2)},
        "decompress": {"ms": round(d_avg, 4), "input_GBps": round(in_bytes / d_avg / 1e6, 1),
                       "elements_per_s": round(n_total / d_avg * 1e3, 0),
                       "pct_hbm_peak": round(100 * alg_bytes / d_avg / 1e6 / HBM_PEAK_GBPS, 2)},
        "fused_pct_hbm_peak": round(100 * 2 * alg_bytes / (c_avg + d_avg) / 1e6 / HBM_PEAK_GBPS, 2),
        "roofline": {"bound": "hbm",
                     "kernel": "gact::multi_inline_kernel<true>" if L <= 64 else "gact::multi_kernel<true>", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": traffic},
    }

    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: the first tensors of the set up to ~cpu_sample_elems elements
        take, acc = [], 0
        for l in range(L):
            take.append(l)
            acc += int(numel[l])
            if acc >= args.cpu_sample_elems:
                break
        host = []
        for l in take:
            t = xs[l]
            host.append(t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16
                        else t.cpu().numpy())
        sample_bytes = sum(h.nbytes for h in host)
        t0 = time.perf_counter()
        comp = [oracle.compress(h, G, int(bits[l]), seeds[l]) for h, l in zip(host, take)]
        t1 = time.perf_counter()
        for (p, mn, sc), h, l in zip(comp, host, take):
            oracle.decompress(p, mn, sc, h.size, G, int(bits[l]),
                              oracle.BF16 if h.dtype == np.uint16 else oracle.F32)
        t2 = time.perf_counter()
        out["cpu_baseline"] = {
            "value": round(2.0 * sample_bytes / (t2 - t0) / 1e9, 3), "unit": "GB/s",
            "cores": oracle.threads(), "kind": "oracle",
            "sample": "first %d tensors of the set (%d elements, %.2f GB), compress %.2f s + decompress %.2f s"
                      % (len(take), acc, sample_bytes / 1e9, t1 - t0, t2 - t1),
        }
    print(json.dumps(out))
    return 0


def bench_grad_sensitivity(args, gact, torch, np, dev) -> int:
    """Alg. 1's reduction 1/2 ||g0 - g1||^2 / S(b) and one running-statistics step
    over a BERT-large-shaped fp32 gradient (391 buffers, 302 M parameters)."""
    shapes = []
    for _ in range(24):
        shapes += [1024 * 1024] * 4 + [1024 * 4096] * 2 + [1024] * 6 + [4096]
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    g0 = [torch.randn(n, device=dev, generator=gen) for n in shapes]
    g1 = [a + 0.01 * torch.randn(n, device=dev, generator=gen) for a, n in zip(g0, shapes)]
    mean = [torch.zeros(n, device=dev) for n in shapes]
    total = sum(shapes)
    ws = torch.empty(gact.gact_reduce_workspace_bytes(len(shapes), total), dtype=torch.uint8, device=dev)
    out1 = torch.empty(1, dtype=torch.float64, device=dev)
    out2 = torch.empty(2, dtype=torch.float64, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    pairs = gact.make_grad_pairs(g0, g1)          # marshalled once, outside the timed region
    stats = gact.make_grad_stats(g0, mean)
    for _ in range(args.warmup):
        gact.gact_sensitivity(g0, g1, 2, out=out1, workspace=ws, pairs=pairs)
        gact.gact_grad_stats_update(g0, mean, 1, out=out2, workspace=ws, stats=stats)
    torch.cuda.synchronize()
    s_ms, u_ms = [], []
    t0 = time.perf_counter()
    marks = []
    for k in range(args.steps):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        gact.gact_sensitivity(g0, g1, 2, out=out1, workspace=ws, pairs=pairs)
        e1.record()
        gact.gact_grad_stats_update(g0, mean, k + 2, out=out2, workspace=ws, stats=stats)
        e2.record()
        marks.append((e0, e1, e2))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for e0, e1, e2 in marks:
        s_ms.append(e0.elapsed_time(e1))
        u_ms.append(e1.elapsed_time(e2))
    s_avg, u_avg = float(np.mean(s_ms)), float(np.mean(u_ms))
    s_bytes, u_bytes = 8 * total, 12 * total        # two reads; two reads + one write
    print(json.dumps({
        "metric": "sensitivity reduction GB/s (bytes read), 1xMI355X", "value": round(s_bytes / s_avg / 1e6, 1),
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall * 1e3 / args.steps, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64 accumulation of f32 inputs", "data": "synthetic",
        "config": {"workload": "grad_sensitivity", "buffers": len(shapes), "elements": total,
                   "description": "BERT-large-shaped fp32 gradient pair; Alg. 1 reduction, then one running-mean step"},
        "sensitivity": {"ms": round(s_avg, 4), "GBps": round(s_bytes / s_avg / 1e6, 1),
                        "pct_hbm_peak": round(100 * s_bytes / s_avg / 1e6 / HBM_PEAK_GBPS, 2)},
        "grad_stats_update": {"ms": round(u_avg, 4), "GBps": round(u_bytes / u_avg / 1e6, 1),
                              "pct_hbm_peak": round(100 * u_bytes / u_avg / 1e6 / HBM_PEAK_GBPS, 2)},
        "roofline": {"bound": "hbm", "kernel": "gact::diff_sq_kernel", "achieved": round(s_bytes / s_avg / 1e6, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(s_bytes / s_avg / 1e6 / HBM_PEAK_GBPS, 4),
                     "traffic": None},
    }))
    return 0


if __name__ == "__main__":
    sys.exit(main())
