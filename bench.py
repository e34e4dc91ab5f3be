#!/usr/bin/env python3
"""Throughput of the GACT compress + decompress hot path on one MI355X.

A step = one pass of the whole path over one synthetic activation set, inputs
already resident in HBM: host bit allocation (Eq. (ilp) of arXiv 2206.11357),
one multi-tensor compress launch, one multi-tensor decompress launch.

Prints ONE JSON line.  The default workload is the largest single-GPU set, the
ViT-L/16-shaped one (400 tensors, bf16, G=128, allocator at 3 bits on average,
32.8 GB of activations).  `value` is uncompressed GB/s averaged over the two
directions: (bytes read by compress + bytes written by decompress) / time.
`roofline` prices the dominant kernel (compress) in algorithmic bytes
(sizeof(T) + bits/8 + 8/G per element) against the 8 TB/s HBM3E peak, with its
launch duration measured by events on the launch stream inside the timed
steps; `roofline.traffic` is the HBM bytes per launch that the FETCH_SIZE and
WRITE_SIZE counters show, taken in two counter passes of this same program
(`--traffic live`, the default: rocprofv3 runs `bench.py --counter-pass` as a
child before this process touches the GPU) and scaled by what the same counters
read for a plain elementwise kernel of known size in the same pass.
`per_config` carries compress / decompress / fused % of peak for the other
benchmark sets (ResNet-50-, BERT-large- and GCN-shaped, and the single 1 Mi
tensor), measured in the same process with fewer repetitions.
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same tensors
on the host cores (all threads, and one thread on a smaller sample); the
oracle's outputs for that sample are also compared with the GPU's, byte for
byte (`parity_checked_elements`).
Also on the line: the same set through one single-tensor call per tensor
(`per_tensor_calls`), a plain device copy's GB/s on the same box
(`copy_ceiling`), what kernels without arithmetic reach for the codec's traffic
mixes (`traffic_ceilings`), and the HBM peak used as denominator.

`--workload single_1m` times the single-tensor calls on 1,048,576 fp32 elements
(launch bound, 4 MiB) over a ring of 128 distinct buffers so that no call finds
its input in a cache.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E, published
# Plain (non-packed, non-matrix) 32-bit vector rate: 256 CUs x 128 lanes x 2.4 GHz, the rate behind the
# published 157.3 TFLOP/s of fp32 vector FMA.  Multiplies, conversions and three-operand integer
# instructions issue at half of it.
VALU_PEAK_LANE_OPS = 256 * 128 * 2.4e9
# VALU instructions per element of the compress kernel, from SQ_INSTS_VALU x 64 / elements (profiles/)
COMPRESS_VALU_PER_ELEMENT = {"f32": 14.9, "bf16": 15.7}

WORKLOADS = {
    # name: (set builder, group size, average bits, sensitivity seed, uniform bits, description)
    "resnet50_b64": ("resnet50_set", 256, 2.0, 2999, False,
                     "53 conv outputs of a ResNet-50-shaped net, batch 64, fp32, G=256, allocator avg 2 bits"),
    "bert_large_b32": ("bert_large_set", 256, 4.0, 3999, False,
                       "96 saved tensors of a BERT-large-shaped encoder, batch 32 x seq 512, bf16, G=256, allocator avg 4 bits"),
    "bert_large_b32_uniform4": ("bert_large_set", 256, 4.0, 3999, True,
                                "96 saved tensors of a BERT-large-shaped encoder, batch 32 x seq 512, bf16, G=256, 4 bits everywhere"),
    "gcn_arxiv": ("gcn_set", 256, 2.0, 4999, True,
                  "3 GCN activations 169343 x 256, fp32, G=256, 2 bits"),
    "gcn_arxiv_b4": ("gcn_set", 256, 4.0, 4999, True,
                     "3 GCN activations 169343 x 256, fp32, G=256, 4 bits"),
    "vit_large_b128": ("vit_large_set", 128, 3.0, 5999, False,
                       "400 saved tensors of a ViT-L/16-shaped model, batch 128, bf16, G=128, allocator avg 3 bits"),
}
DEFAULT_WORKLOAD = "vit_large_b128"          # the largest single-GPU configuration
PER_CONFIG = ("resnet50_b64", "bert_large_b32", "bert_large_b32_uniform4", "gcn_arxiv", "gcn_arxiv_b4")
ESIZE = {"f32": 4, "bf16": 2}


class ActivationSet:
    """One benchmark set resident on the device: inputs, output buffers, launch descriptors."""

    def __init__(self, workload, gact, torch, np, syn, dev):
        builder, self.G, self.avg_bits, sens_seed, uniform, self.desc = WORKLOADS[workload]
        self.workload, self.gact, self.torch, self.np = workload, gact, torch, np
        self.specs = getattr(syn, builder)()
        self.L = len(self.specs)
        self.numel = np.array([s.numel for s in self.specs], dtype=np.int64)
        self.sens = syn.lognormal_sensitivities(self.L, sens_seed)
        if uniform:
            self.sens[:] = 1.0                  # the same width everywhere
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16}
        self.xs = [syn.draw_torch(s, dev) for s in self.specs]
        self.bits = gact.gact_allocate_bits(self.sens, self.numel, self.avg_bits)
        # buffers sized for the widest code so that any allocation result fits
        self.packed, self.gmin, self.gscale, self.ys = [], [], [], []
        for s, x in zip(self.specs, self.xs):
            p, mn, sc = gact.alloc_compressed(s.numel, self.G, 8, dev)
            self.packed.append(p); self.gmin.append(mn); self.gscale.append(sc)
            self.ys.append(torch.empty_like(x))
        self.ws = torch.empty(gact.gact_multi_workspace_bytes(self.L), dtype=torch.uint8, device=dev)
        self.seeds = [s.seed for s in self.specs]
        self.dts = [tdt[s.dtype] for s in self.specs]
        self.n_total = int(self.numel.sum())
        self.in_bytes = int(sum(int(n) * ESIZE[s.dtype] for n, s in zip(self.numel, self.specs)))
        packed_bytes = int(sum(gact.gact_packed_bytes(int(n), int(b)) for n, b in zip(self.numel, self.bits)))
        meta_bytes = int(sum(8 * gact.gact_num_groups(int(n), self.G) for n in self.numel))
        self.alg_bytes = self.in_bytes + packed_bytes + meta_bytes          # per direction
        torch.cuda.synchronize()

    def step(self, record: bool):
        """Host allocation + one launch per direction; returns the three events when recording."""
        g, torch = self.gact, self.torch
        b = g.gact_allocate_bits(self.sens, self.numel, self.avg_bits)
        descs = g.make_descs(self.xs, self.packed, self.gmin, self.gscale, self.ys, self.numel, b,
                             self.seeds, self.dts)
        if record:
            e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            e0.record()
        g.gact_compress_multi(descs, self.L, self.G, self.ws)
        if record:
            e1.record()
        g.gact_decompress_multi(descs, self.L, self.G, self.ws)
        if record:
            e2.record()
            return e0, e1, e2
        return None

    def timed(self, steps: int, warmup: int):
        """-> (compress ms list, decompress ms list, wall seconds of the `steps` steps)"""
        torch = self.torch
        for _ in range(warmup):
            self.step(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks = [self.step(True) for _ in range(steps)]
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return ([a.elapsed_time(b) for a, b, _ in marks], [b.elapsed_time(c) for _, b, c in marks], wall)

    def per_tensor(self, reps: int):
        """The set through one single-tensor call per tensor and direction -> median ms each way."""
        g, torch, np = self.gact, self.torch, self.np
        out = []
        for rep in range(reps + 1):
            e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            stream = torch.cuda.current_stream().cuda_stream       # resolved once per sweep
            e0.record()
            for l in range(self.L):
                g.gact_compress(self.xs[l], self.G, int(self.bits[l]), self.seeds[l], self.packed[l],
                                self.gmin[l], self.gscale[l], stream)
            e1.record()
            for l in range(self.L):
                g.gact_decompress(self.packed[l], self.gmin[l], self.gscale[l], int(self.numel[l]), self.G,
                                  int(self.bits[l]), self.dts[l], self.ys[l], stream)
            e2.record()
            torch.cuda.synchronize()
            if rep:                              # the first sweep is a warm-up
                out.append((e0.elapsed_time(e1), e1.elapsed_time(e2)))
        return float(np.median([a for a, _ in out])), float(np.median([b for _, b in out]))

    def direction(self, ms_list):
        np = self.np
        avg = float(np.mean(ms_list))
        return {"ms": round(avg, 4), "ms_median": round(float(np.median(ms_list)), 4),
                "ms_min": round(float(np.min(ms_list)), 4), "input_GBps": round(self.in_bytes / avg / 1e6, 1),
                "elements_per_s": round(self.n_total / avg * 1e3, 0),
                "pct_hbm_peak": round(100 * self.alg_bytes / avg / 1e6 / HBM_PEAK_GBPS, 2)}

    def fused_pct(self, c_ms, d_ms):
        np = self.np
        return round(100 * 2 * self.alg_bytes / (float(np.mean(c_ms)) + float(np.mean(d_ms))) / 1e6 / HBM_PEAK_GBPS, 2)

    def release(self):
        self.xs = self.packed = self.gmin = self.gscale = self.ys = self.ws = None
        self.torch.cuda.empty_cache()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD,
                    choices=sorted(WORKLOADS) + ["grad_sensitivity", "single_1m", "hooks_transformer", "fused_footprint"])
    ap.add_argument("--swap-workgroups", type=int, default=16,
                    help="hooks_transformer: workgroups of the kernel that copies compressed batches to the host")
    ap.add_argument("--prefetch-batches", type=int, default=8,
                    help="hooks_transformer: swapped batches fetched ahead of use in the backward pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="skip the other benchmark sets")
    ap.add_argument("--cpu-sample-elems", type=int, default=1_400_000_000)
    ap.add_argument("--traffic", choices=("live", "profile", "off"), default="live",
                    help="roofline.traffic from two rocprofv3 counter passes of this program run now (live), "
                         "from the committed summaries under profiles/ (profile), or null (off)")
    ap.add_argument("--counter-pass", action="store_true",
                    help="child mode of --traffic live: a reference kernel of known size, then two launches "
                         "per direction of the workload, nothing else")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the workload, launch a plain elementwise kernel that reads "
                         "1 GiB and writes 1 GiB five times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no cross-GPU step and this build runs on "
              "single-GPU boxes; run with --gpus 1", file=sys.stderr)
        return 2

    is_set = args.workload in WORKLOADS and not args.copy_calibration
    # Both are programs of their own: they run, and end, before this process touches the GPU.
    ceilings = traffic_ceilings() if is_set and not args.counter_pass else None
    traffic = None
    if is_set and not args.counter_pass:
        if args.traffic == "live":
            traffic = live_traffic(args.workload)
        if args.traffic == "profile" or (args.traffic == "live" and traffic is None):
            traffic = profile_traffic(args.workload)

    import numpy as np
    import torch
    import paper_2206_11357_amd as gact
    import synthetic_inputs as syn

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.copy_calibration or args.counter_pass:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5 if args.copy_calibration else 3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        info = {"copy_calibration": True, "kernel": "torch.add(src, 1.0, out=dst)",
                "read_bytes_per_launch": src.numel() * 4, "write_bytes_per_launch": dst.numel() * 4}
        if args.copy_calibration:
            print(json.dumps(dict(info, launches=5)))
            return 0
        del src, dst
        S = ActivationSet(args.workload, gact, torch, np, syn, dev)
        for _ in range(2):
            S.step(False)
        torch.cuda.synchronize()
        print(json.dumps(dict(info, counter_pass=True, workload=args.workload,
                              algorithmic_bytes_per_direction=S.alg_bytes)))
        return 0

    if args.workload == "grad_sensitivity":
        return bench_grad_sensitivity(args, gact, torch, np, dev)
    if args.workload == "single_1m":
        print(json.dumps(bench_single_1m(args.steps, args.warmup, gact, torch, np, dev)))
        return 0
    if args.workload == "hooks_transformer":
        return bench_hooks_transformer(args, gact, torch, np, dev)
    if args.workload == "fused_footprint":
        return bench_fused_footprint(args, gact, torch, np, dev)

    # inputs resident in HBM before anything is timed
    S = ActivationSet(args.workload, gact, torch, np, syn, dev)
    L, G = S.L, S.G

    # Side measurements first (they also bring the GPU to its working clocks): the same set with one
    # single-tensor call per tensor and direction, and a plain device copy.
    pt_reps = max(args.steps // 4, 3)
    pt_c, pt_d = S.per_tensor(pt_reps)
    copy_info = copy_ceiling(torch, np, dev)

    # the timed steps
    c_ms, d_ms, wall = S.timed(args.steps, args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    c_avg, d_avg = float(np.mean(c_ms)), float(np.mean(d_ms))
    value = 2.0 * S.in_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = S.alg_bytes / (c_avg * 1e-3) / 1e9
    achieved_d = S.alg_bytes / (d_avg * 1e-3) / 1e9
    kernel = "gact::multi_inline_kernel<%s>" if L <= 64 else "gact::multi_kernel<%s>"
    valu = COMPRESS_VALU_PER_ELEMENT[S.specs[0].dtype] * S.n_total / c_avg * 1e3

    roof = {"bound": "hbm", "kernel": kernel % "true", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": traffic["compress_bytes"] if traffic else None}
    roof_d = {"bound": "hbm", "kernel": kernel % "false", "achieved": round(achieved_d, 1), "peak": HBM_PEAK_GBPS,
              "unit": "GB/s", "frac": round(achieved_d / HBM_PEAK_GBPS, 4),
              "traffic": traffic["decompress_bytes"] if traffic else None}
    if traffic:
        roof["traffic_over_algorithmic"] = round(traffic["compress_bytes"] / S.alg_bytes, 4)
        roof_d["traffic_over_algorithmic"] = round(traffic["decompress_bytes"] / S.alg_bytes, 4)
        roof["traffic_source"] = roof_d["traffic_source"] = traffic["source"]

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
        "dtype": S.specs[0].dtype,
        "data": "synthetic",
        "config": {
            "workload": args.workload, "description": S.desc, "tensors": L, "elements": S.n_total,
            "group_size": G, "avg_bits": S.avg_bits,
            "bits_histogram": {str(k): int((S.bits == k).sum()) for k in (1, 2, 4, 8)},
            "input_bytes": S.in_bytes, "algorithmic_bytes_per_direction": S.alg_bytes,
            "launch": "one multi-tensor launch per direction",
        },
        "pre_timed_work": "before the %d warm-up steps this process ran %d sweeps of single-tensor calls over the set "
                          "and 13 device copies of 1 GiB (the side measurements below), so the timed steps start "
                          "with the GPU at its working clocks" % (args.warmup, pt_reps + 1),
        "compress": S.direction(c_ms),
        "decompress": S.direction(d_ms),
        "fused_pct_hbm_peak": S.fused_pct(c_ms, d_ms),
        "roofline": roof,
        "roofline_decompress": roof_d,
        "roofline_alu": {"bound": "alu", "kernel": "compress", "achieved": round(valu, 0),
                         "peak": VALU_PEAK_LANE_OPS, "unit": "lane-ops/s", "frac": round(valu / VALU_PEAK_LANE_OPS, 4),
                         "note": "secondary bound; about half of the instruction mix issues at half rate"},
        "per_tensor_calls": {"calls_per_direction": L, "compress_ms": round(pt_c, 4), "decompress_ms": round(pt_d, 4),
                             "fused_pct_hbm_peak": round(100 * 2 * S.alg_bytes / (pt_c + pt_d) / 1e6 / HBM_PEAK_GBPS, 2)},
        "copy_ceiling": copy_info,
        "traffic_ceilings": ceilings,
        "hbm_peak": hbm_peak_info(torch),
    }
    if traffic and traffic.get("detail"):
        out["traffic_detail"] = traffic["detail"]

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(S, args.cpu_sample_elems, torch, np)
        out["parity_checked_elements"] = out["cpu_baseline"].pop("parity_checked_elements")

    if not args.no_per_config:
        S.release()
        del S
        per = {}
        k_steps, k_warm = max(args.steps, 10), 5
        for w in PER_CONFIG:
            if w == args.workload:
                continue
            T = ActivationSet(w, gact, torch, np, syn, dev)
            tc, td, _ = T.timed(k_steps, k_warm)
            per[w] = {"description": T.desc, "dtype": T.specs[0].dtype, "tensors": T.L, "input_bytes": T.in_bytes,
                      "algorithmic_bytes_per_direction": T.alg_bytes, "steps": k_steps, "warmup": k_warm,
                      "compress_ms": round(float(np.mean(tc)), 4), "decompress_ms": round(float(np.mean(td)), 4),
                      "compress_pct_hbm_peak": T.direction(tc)["pct_hbm_peak"],
                      "decompress_pct_hbm_peak": T.direction(td)["pct_hbm_peak"],
                      "fused_pct_hbm_peak": T.fused_pct(tc, td)}
            T.release()
            del T
        one = bench_single_1m(k_steps, k_warm, gact, torch, np, dev)
        per["single_1m"] = {"description": one["config"]["description"], "dtype": "f32",
                            "compress_us_per_call": one["compress"]["us_per_call_median"],
                            "decompress_us_per_call": one["decompress"]["us_per_call_median"],
                            "compress_pct_hbm_peak": one["compress"]["pct_hbm_peak"],
                            "decompress_pct_hbm_peak": one["decompress"]["pct_hbm_peak"],
                            "fused_pct_hbm_peak": round(2 / (1 / max(one["compress"]["pct_hbm_peak"], 1e-9)
                                                             + 1 / max(one["decompress"]["pct_hbm_peak"], 1e-9)), 2),
                            "note": "launch bound: 4.5 MB per call"}
        out["per_config"] = per
    print(json.dumps(out))
    return 0


def cpu_baseline(S, sample_elems, torch, np) -> dict:
    """The oracle on a bounded sample (the first tensors of the set up to about `sample_elems`
    elements) on all host threads, and on one thread on a smaller sample.  The GPU buffers of the
    sampled tensors, left by the last timed step, are compared byte for byte with the oracle's."""
    import oracle
    take, acc = [], 0
    for l in range(S.L):
        take.append(l)
        acc += int(S.numel[l])
        if acc >= sample_elems:
            break

    def host(t):
        return t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.cpu().numpy()
    xs = [host(S.xs[l]) for l in take]
    sample_bytes = sum(h.nbytes for h in xs)
    t0 = time.perf_counter()
    comp = [oracle.compress(h, S.G, int(S.bits[l]), S.seeds[l]) for h, l in zip(xs, take)]
    t1 = time.perf_counter()
    ys = [oracle.decompress(p, mn, sc, h.size, S.G, int(S.bits[l]), oracle.BF16 if h.dtype == np.uint16 else oracle.F32)
          for (p, mn, sc), h, l in zip(comp, xs, take)]
    t2 = time.perf_counter()
    checked, mismatches = 0, []
    for (p, mn, sc), y, l in zip(comp, ys, take):
        ok = (np.array_equal(S.packed[l][:p.size].cpu().numpy(), p)
              and np.array_equal(S.gmin[l].cpu().numpy().view(np.uint32), mn.view(np.uint32))
              and np.array_equal(S.gscale[l].cpu().numpy().view(np.uint32), sc.view(np.uint32))
              and np.array_equal(host(S.ys[l]).view(np.uint16 if y.dtype == np.uint16 else np.uint32),
                                 y.view(np.uint16 if y.dtype == np.uint16 else np.uint32)))
        checked += int(S.numel[l])
        if not ok:
            mismatches.append(S.specs[l].name)
    if mismatches:
        raise SystemExit("bench.py: GPU output differs from the oracle on %s" % ", ".join(mismatches[:8]))
    all_threads = oracle.threads()
    # one thread, on the first 32 Mi elements of the first tensor
    h1 = xs[0][: 1 << 25]
    oracle.set_threads(1)
    t3 = time.perf_counter()
    p1, mn1, sc1 = oracle.compress(h1, S.G, int(S.bits[take[0]]), S.seeds[take[0]])
    oracle.decompress(p1, mn1, sc1, h1.size, S.G, int(S.bits[take[0]]),
                      oracle.BF16 if h1.dtype == np.uint16 else oracle.F32)
    t4 = time.perf_counter()
    oracle.set_threads(all_threads)
    classes = sorted({S.specs[l].name.split(".")[-1].rstrip("0123456789") for l in take})
    return {
        "value": round(2.0 * sample_bytes / (t2 - t0) / 1e9, 3), "unit": "GB/s",
        "cores": all_threads, "kind": "oracle",
        "compress_GBps": round(sample_bytes / (t1 - t0) / 1e9, 3),
        "decompress_GBps": round(sample_bytes / (t2 - t1) / 1e9, 3),
        "sample": "first %d of %d tensors of the set (shape classes %s; %d elements, %.2f GB), compress %.2f s + "
                  "decompress %.2f s; the rate stands for the whole set (extrapolated by element count)"
                  % (len(take), S.L, "/".join(classes), acc, sample_bytes / 1e9, t1 - t0, t2 - t1),
        "value_1_thread": round(2.0 * h1.nbytes / (t4 - t3) / 1e9, 3),
        "sample_1_thread": "first %d elements of the first tensor, %.2f s" % (h1.size, t4 - t3),
        "parity_checked_elements": checked,
    }


# ----------------------------------------------------------------- HBM traffic from counters
TRAFFIC_COUNTERS = ("FETCH_SIZE", "WRITE_SIZE")        # KiB per dispatch


def _counter_rows(csv_path):
    import csv
    with open(csv_path, newline="") as f:
        for r in csv.DictReader(f):
            yield r["Kernel_Name"], r["Counter_Name"], float(r["Counter_Value"])


def live_traffic(workload: str):
    """HBM bytes per compress / decompress launch from two rocprofv3 counter passes of this
    program (`--counter-pass`), each scaled by what the same counter reads, in the same pass, for an
    elementwise kernel that reads 1 GiB and writes 1 GiB.  None when a pass cannot be taken."""
    import glob
    import shutil
    import signal
    import subprocess
    import tempfile
    exe = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(exe):
        return None
    out_dir = tempfile.mkdtemp(prefix="gact_traffic_", dir="/tmp")
    env = dict(os.environ, TMPDIR="/tmp")
    gib = float(1 << 30)
    res, detail = {}, {}
    try:
        for counter in TRAFFIC_COUNTERS:
            cmd = [exe, "--pmc", counter, "--output-format", "csv", "-d", out_dir, "-o", counter.lower(), "--",
                   sys.executable, os.path.join(ROOT, "bench.py"), "--counter-pass", "--workload", workload]
            p = subprocess.Popen(cmd, cwd="/tmp", env=env, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL,
                                 start_new_session=True)
            try:
                rc = p.wait(timeout=240)
            except subprocess.TimeoutExpired:
                os.killpg(p.pid, signal.SIGKILL)
                p.wait()
                return None
            if rc != 0:
                return None
            files = glob.glob(os.path.join(out_dir, "**", "%s_counter_collection.csv" % counter.lower()), recursive=True)
            if not files:
                return None
            ref, comp, dec = [], [], []
            for name, cname, val in _counter_rows(files[0]):
                if cname != counter:
                    continue
                if "vectorized_elementwise_kernel" in name and "_add<" in name and val > 100000:      # the reference kernel
                    ref.append(val)
                elif "gact::multi" in name and "<true>" in name:
                    comp.append(val)
                elif "gact::multi" in name and "<false>" in name:
                    dec.append(val)
            if not ref or not comp or not dec:
                return None
            scale = gib / (sum(ref) / len(ref) * 1024.0)        # true bytes per counted byte
            res[counter] = (scale * 1024.0 * sum(comp) / len(comp), scale * 1024.0 * sum(dec) / len(dec))
            detail[counter] = {"reference_KiB_for_1GiB": round(sum(ref) / len(ref), 1), "scale": round(scale, 4),
                               "compress_KiB": round(sum(comp) / len(comp), 1), "decompress_KiB": round(sum(dec) / len(dec), 1),
                               "launches": len(comp)}
    except Exception:                                            # measurement aid only
        return None
    finally:
        shutil.rmtree(out_dir, ignore_errors=True)
    return {"compress_bytes": int(res["FETCH_SIZE"][0] + res["WRITE_SIZE"][0]),
            "decompress_bytes": int(res["FETCH_SIZE"][1] + res["WRITE_SIZE"][1]),
            "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes of `bench.py --counter-pass` in this run",
            "detail": detail}


def profile_traffic(workload: str):
    """The figures of the committed counter summaries under profiles/ (None if the workload has none)."""
    import re
    found = {}
    try:
        for name in sorted(os.listdir(os.path.join(ROOT, "profiles"))):
            text = open(os.path.join(ROOT, "profiles", name)).read()
            for kind in ("compress", "decompress"):
                m = re.search(r"traffic_%s_bytes_per_launch\[%s\]\s*=\s*(\d+)" % (kind, re.escape(workload)), text)
                if m:
                    found[kind] = int(m.group(1))
    except OSError:
        return None
    if "compress" not in found or "decompress" not in found:
        return None
    return {"compress_bytes": found["compress"], "decompress_bytes": found["decompress"],
            "source": "committed summary under profiles/ (not measured in this run)", "detail": None}


def copy_ceiling(torch, np, dev) -> dict:
    """A plain device-to-device copy of 1 GiB on this machine: GB/s in read + written bytes."""
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    ms = []
    for _ in range(10):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(); dst.copy_(src); b.record(); b.synchronize()
        ms.append(a.elapsed_time(b))
    m = float(np.median(ms))
    return {"kernel": "torch copy_ of 1 GiB", "GBps_read_plus_write": round(2 * src.numel() * 4 / m / 1e6, 1),
            "pct_hbm_peak": round(100 * 2 * src.numel() * 4 / m / 1e6 / HBM_PEAK_GBPS, 2)}


def traffic_ceilings():
    """What kernels without arithmetic reach on this machine for the codec's traffic mixes (same access
    shape: 8 KB per wavefront in coalesced 16-byte non-temporal accesses, 512 B the other way):
    the memory system's own limit next to which `roofline.achieved` should be read.  None when the
    probe has not been built."""
    import subprocess
    exe = os.path.join(ROOT, "paper_2206_11357_amd", "traffic_probe.bin")
    if not os.path.exists(exe):
        return None
    try:
        r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
        if r.returncode != 0:
            return {"error": r.stderr.strip()[-200:]}
        out = json.loads(r.stdout.strip().splitlines()[-1])
        for k in list(out):
            if k.endswith("_GBps"):
                out[k.replace("_GBps", "_pct_hbm_peak")] = round(100 * out[k] / HBM_PEAK_GBPS, 1)
        return out
    except Exception as e:                                   # measurement aid only
        return {"error": str(e)[-200:]}


def hbm_peak_info(torch) -> dict:
    """The denominator used, and what the device properties give (clock x bus width x 2)."""
    info = {"used_GBps": HBM_PEAK_GBPS, "source": "published MI355X HBM3E bandwidth"}
    try:
        p = torch.cuda.get_device_properties(0)
        khz, width = getattr(p, "memory_clock_rate", None), getattr(p, "memory_bus_width", None)
        if khz and width:
            info["device_props_GBps"] = round(2.0 * khz * 1e3 * width / 8 / 1e9, 1)
            info["memory_clock_khz"], info["memory_bus_width_bits"] = int(khz), int(width)
        info["device"] = p.name
    except Exception as e:                                   # properties missing on this build
        info["device_props_error"] = str(e)
    return info


def bench_single_1m(steps, warmup, gact, torch, np, dev) -> dict:
    """Single-tensor calls on 1,048,576 fp32 elements (N(0,1), 1 % outliers x10), G=256, 2 bits,
    over a ring of 128 distinct buffers (512 MiB of inputs) so that no call is served from a cache."""
    import synthetic_inputs as syn
    ring, n, G, b = 128, 1 << 20, 256, 2
    base = torch.from_numpy(syn.config1()["x"]).to(dev)
    xs = [base.clone().mul_(1.0 + 0.001 * k) for k in range(ring)]
    bufs = [gact.alloc_compressed(n, G, b, dev) for _ in range(ring)]
    ys = [torch.empty_like(x) for x in xs]
    ev = lambda: torch.cuda.Event(enable_timing=True)
    cs = [gact.prepare_compress(xs[k], G, b, 0, *bufs[k]) for k in range(ring)]
    ds = [gact.prepare_decompress(*bufs[k], n, G, b, ys[k]) for k in range(ring)]

    def sweep(record):
        e0, e1, e2 = ev(), ev(), ev()
        stream = torch.cuda.current_stream().cuda_stream
        if record: e0.record()
        for k in range(ring):
            cs[k](stream)
        if record: e1.record()
        for k in range(ring):
            ds[k](stream)
        if record: e2.record()
        return e0, e1, e2
    for _ in range(warmup):
        sweep(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks = [sweep(True) for _ in range(steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    c_us = np.array([a.elapsed_time(b) for a, b, _ in marks]) * 1e3 / ring
    d_us = np.array([b.elapsed_time(c) for _, b, c in marks]) * 1e3 / ring
    alg = n * 4 + n * b // 8 + (n // G) * 8
    cm, dm = float(np.median(c_us)), float(np.median(d_us))
    return {
        "metric": "compress+decompress GB/s (input bytes) and % of HBM peak, 1xMI355X",
        "value": round(2 * n * 4 / ((cm + dm) * 1e-6) / 1e9, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(wall * 1e3 / steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "single_1m", "elements": n, "group_size": G, "bits": b, "ring_buffers": ring,
                   "description": "one step = 128 compress calls then 128 decompress calls (prepared-call objects), each on "
                                  "its own 4 MiB fp32 tensor, G=256, 2 bits; back-to-back launches on one stream, so the "
                                  "per-call time is the launch-bound issue rate"},
        "compress": {"us_per_call_median": round(cm, 2), "us_per_call_min": round(float(c_us.min()), 2),
                     "pct_hbm_peak": round(100 * alg / cm / 1e3 / HBM_PEAK_GBPS, 2)},
        "decompress": {"us_per_call_median": round(dm, 2), "us_per_call_min": round(float(d_us.min()), 2),
                       "pct_hbm_peak": round(100 * alg / dm / 1e3 / HBM_PEAK_GBPS, 2)},
        "roofline": {"bound": "hbm", "kernel": "gact::single_kernel<true>", "achieved": round(alg / cm / 1e3, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(alg / cm / 1e3 / HBM_PEAK_GBPS, 4),
                     "traffic": None},
    }


def bench_hooks_transformer(args, gact, torch, np, dev) -> int:
    """Training steps of a small pre-LN transformer encoder (8 layers, hidden 1024, 16 heads, FFN 4096,
    batch 16 x 512 tokens, bf16 autocast-free: parameters and activations in bf16) with autograd's saved
    tensors routed through the compressor (Sec. 5 hook interface): peak memory and step time without
    hooks, with 4-bit and 2-bit compression (the paper's L1-type levels), and with the compressed tensors
    swapped to pinned host memory (L2-type)."""
    from paper_2206_11357_amd.hooks import Controller
    nn = torch.nn
    H, heads, F, layers, B, S = 1024, 16, 4096, 8, 16, 512

    class Block(nn.Module):
        def __init__(self):
            super().__init__()
            self.ln1, self.ln2 = nn.LayerNorm(H), nn.LayerNorm(H)
            self.qkv, self.proj = nn.Linear(H, 3 * H), nn.Linear(H, H)
            self.fc1, self.fc2 = nn.Linear(H, F), nn.Linear(F, H)

        def forward(self, x):
            h = self.ln1(x)
            q, k, v = self.qkv(h).view(B, S, 3, heads, H // heads).permute(2, 0, 3, 1, 4)
            att = torch.softmax((q @ k.transpose(-1, -2)) * (H // heads) ** -0.5, dim=-1)
            x = x + self.proj((att @ v).transpose(1, 2).reshape(B, S, H))
            return x + self.fc2(nn.functional.gelu(self.fc1(self.ln2(x))))

    torch.manual_seed(0)
    model = nn.Sequential(*[Block() for _ in range(layers)]).to(dev).to(torch.bfloat16)
    opt = torch.optim.SGD(model.parameters(), lr=1e-3)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    x = torch.randn(B, S, H, device=dev, dtype=torch.bfloat16, generator=gen)
    target = torch.randn(B, S, H, device=dev, dtype=torch.bfloat16, generator=gen)

    def run(ctl, steps, warmup):
        def one():
            opt.zero_grad(set_to_none=True)
            if ctl is None:
                loss = (model(x) - target).float().pow(2).mean()
            else:
                ctl.begin_iteration()
                with ctl.hooks():
                    loss = (model(x) - target).float().pow(2).mean()
            loss.backward()
            opt.step()
            return loss
        for _ in range(warmup):
            one()
        torch.cuda.synchronize()
        if ctl is not None:
            ctl.release()                    # the last warm-up step's compressed buffers are not part of the base
        torch.cuda.reset_peak_memory_stats()
        base = torch.cuda.memory_allocated()
        t0 = time.perf_counter()
        for _ in range(steps):
            loss = one()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        return {"ms_per_step": round(dt * 1e3, 2), "loss": round(float(loss.detach()), 5),
                "peak_activation_MB": round((torch.cuda.max_memory_allocated() - base) / 2**20, 1),
                "compressed_MB": None if ctl is None else round(sum(b.nbytes for b in ctl._batches) / 2**20, 1),
                "swapped_MB": None if ctl is None else round(sum(b.nbytes for b in ctl._batches if b.host is not None) / 2**20, 1)}

    steps, warmup = max(args.steps // 4, 3), max(args.warmup, 2)
    params = list(model.parameters())
    res = {"no_hooks": run(None, steps, warmup)}
    wg, pf = args.swap_workgroups, args.prefetch_batches

    def level(bits, **kw):
        ctl = Controller(params, group_size=256, bits=bits, seed=0, min_numel=1 << 14, swap_workgroups=wg,
                         prefetch_batches=pf, **kw)
        out = run(ctl, steps, warmup)
        # the next level starts from an empty allocator cache: blocks that a level leaves waiting on its
        # side streams slowed the levels after it by up to 5 ms per step
        del ctl
        gc.collect()
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        return out
    res["compress_4bit_no_dedup"] = level(4)
    res["compress_4bit"] = level(4, dedup=True)
    res["compress_2bit"] = level(2, dedup=True)
    # bits from the paper's adaptive algorithm: sensitivities by Alg. 1 (L + 1 seeded passes on this batch),
    # widths by Eq. (ilp) at an average of 3 bits
    ctl = Controller(params, group_size=256, bits=4, seed=0, min_numel=1 << 14, dedup=True)

    def fwdbwd():
        opt.zero_grad(set_to_none=True)
        with ctl.hooks():
            loss = (model(x) - target).float().pow(2).mean()
        loss.backward()
        return [p.grad for p in params]
    t0 = time.perf_counter()
    sens = ctl.compute_sensitivities(fwdbwd)
    adapted = ctl.adapt(3.0)
    torch.cuda.synchronize()
    t_adapt = time.perf_counter() - t0
    res["compress_adaptive_avg3"] = run(ctl, steps, warmup)
    res["compress_adaptive_avg3"].update({
        "context_tensors": int(len(adapted)), "adapt_seconds": round(t_adapt, 2),
        "bits_histogram": {str(k): int((adapted == k).sum()) for k in (1, 2, 4, 8)},
        "sensitivity_min_max": [float(sens.min()), float(sens.max())]})
    del ctl
    gc.collect()
    torch.cuda.empty_cache()
    res["compress_4bit_swap"] = level(4, dedup=True, swap=True)
    res["compress_4bit_swap_inflight_4"] = level(4, dedup=True, swap=True, swap_inflight_batches=4)
    res["compress_4bit_swap_inflight_12"] = level(4, dedup=True, swap=True, swap_inflight_batches=12)
    res["compress_2bit_swap"] = level(2, dedup=True, swap=True)
    res["compress_4bit_swap_strict"] = level(4, dedup=True, swap=True, keep_until_copied=False)
    ref = res["no_hooks"]
    for k, r in res.items():
        r["activation_memory_ratio"] = round(ref["peak_activation_MB"] / max(r["peak_activation_MB"], 1e-9), 2)
        r["step_time_ratio"] = round(r["ms_per_step"] / ref["ms_per_step"], 3)
    print(json.dumps({
        "metric": "peak activation memory reduction of a training step with saved tensors compressed, 1xMI355X",
        "value": res["compress_4bit"]["activation_memory_ratio"], "unit": "x", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": res["compress_4bit"]["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "hooks_transformer", "layers": layers, "hidden": H, "heads": heads, "ffn": F,
                   "batch": B, "seq_len": S, "group_size": 256, "swap_workgroups": wg, "prefetch_batches": pf,
                   "description": "pre-LN encoder with explicit softmax attention, SGD, MSE loss on random data; "
                                  "peak memory above what is allocated before the step"},
        "levels": res,
    }))
    return 0


def bench_fused_footprint(args, gact, torch, np, dev) -> int:
    """The compressor with the duplicate footprint (Sec. 5.2) taken in its statistics pass, against
    the plain compressor and against compressor + separate footprint pass: one tensor of 2^29 fp32
    elements, G=256, 2 bits, 8 sampled points."""
    n, G, b, ns = 1 << 29, 256, 2, 8
    gen = torch.Generator(device=dev)
    gen.manual_seed(3)
    x = torch.randn(n, device=dev, generator=gen).relu_()
    p, mn, sc = gact.alloc_compressed(n, G, b, dev)
    fp = torch.empty(1 + ns, dtype=torch.float64, device=dev)
    ws = torch.empty(gact.gact_compress_footprint_workspace_bytes(n, G), dtype=torch.uint8, device=dev)
    ws2 = torch.empty(gact.gact_reduce_workspace_bytes(1, n), dtype=torch.uint8, device=dev)
    calls = {"compress": lambda: gact.gact_compress(x, G, b, 1, p, mn, sc),
             "footprint": lambda: gact.gact_footprint(x, ns, fp, ws2),
             "compress_footprint": lambda: gact.gact_compress_footprint(x, G, b, 1, ns, p, mn, sc, fp, ws)}
    ms = {}
    t0 = time.perf_counter()
    for name, f in calls.items():
        for _ in range(args.warmup):
            f()
        torch.cuda.synchronize()
        t = []
        for _ in range(args.steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); f(); e1.record(); e1.synchronize()
            t.append(e0.elapsed_time(e1))
        ms[name] = float(np.median(t))
    wall = time.perf_counter() - t0
    alg = n * 4 + n * b // 8 + (n // G) * 8 + (n // 2048) * 8          # + one partial sum per tile
    print(json.dumps({
        "metric": "compress with fused footprint, algorithmic GB/s, 1xMI355X",
        "value": round(alg / ms["compress_footprint"] / 1e6, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall * 1e3 / (3 * args.steps), 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "fused_footprint", "elements": n, "group_size": G, "bits": b, "n_samples": ns},
        "ms": {k: round(v, 4) for k, v in ms.items()},
        "separate_passes_ms": round(ms["compress"] + ms["footprint"], 4),
        "roofline": {"bound": "hbm", "kernel": "gact::compress_sum_kernel",
                     "achieved": round(alg / ms["compress_footprint"] / 1e6, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(alg / ms["compress_footprint"] / 1e6 / HBM_PEAK_GBPS, 4),
                     "traffic": None},
    }))
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
