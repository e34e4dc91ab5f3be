"""Seeded synthetic activation tensors, shared by the tests, the smoke check and
the benchmark.  Holds no arithmetic of the compression method: it only draws
values with the shapes and distributions of the paper's CNN / transformer /
GNN workloads (arXiv 2206.11357, Sec. 6: ResNet-50, BERT-large, GCN on a
169,343-node graph, ViT-class models) and converts dtypes.

Small tensors come from numpy's ``default_rng``; the large activation sets are
described by ``TensorSpec`` records and materialised on a torch device with a
seeded ``torch.Generator``.  bf16 tensors are handed to numpy consumers as
``uint16`` bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

# value laws
NORMAL = "normal"            # N(0,1)
RELU = "relu"                # max(N(0,1), 0): half exact zeros
GELU = "gelu"                # gelu(N(0,1))
SOFTMAX = "softmax"          # softmax(2*N(0,1)) along rows of `row` elements
OUTLIER = "outlier"          # N(0,1), 1% of positions multiplied by 10


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: tuple
    law: str
    dtype: str               # "f32" | "bf16"
    data_seed: int
    seed: int                # compressor seed (the paper's r_l)
    row: int = 0             # softmax row length

    @property
    def numel(self) -> int:
        n = 1
        for s in self.shape:
            n *= s
        return n


# ----------------------------------------------------------------- numpy side
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 array of bf16 bit patterns (round-nearest-even),
    through torch's CPU cast so that no rounding code is written here."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (h.astype(np.uint32) << 16).view(np.float32)


def draw_numpy(law: str, n: int, data_seed: int, row: int = 0) -> np.ndarray:
    """float32 vector of n values under `law`."""
    rng = np.random.default_rng(data_seed)
    if law == NORMAL:
        return rng.standard_normal(n, dtype=np.float32)
    if law == RELU:
        return np.maximum(rng.standard_normal(n, dtype=np.float32), np.float32(0))
    if law == OUTLIER:
        x = rng.standard_normal(n, dtype=np.float32)
        k = max(n // 100, 1) if n >= 1 else 0
        pos = rng.choice(n, size=k, replace=False) if n else np.empty(0, dtype=np.int64)
        x[pos] *= np.float32(10)
        return x
    if law == GELU:
        import torch
        z = torch.from_numpy(rng.standard_normal(n, dtype=np.float32))
        return torch.nn.functional.gelu(z).numpy()
    if law == SOFTMAX:
        import torch
        assert row > 0 and n % row == 0
        z = torch.from_numpy(rng.standard_normal(n, dtype=np.float32)).view(-1, row)
        return torch.softmax(z * 2.0, dim=-1).reshape(-1).numpy()
    raise ValueError(law)


def config1() -> dict:
    """Single fp32 tensor: 1,048,576 elements ~N(0,1) with 1% outliers x10,
    group_size=256, bits=2, seed=0."""
    return dict(x=draw_numpy(OUTLIER, 1 << 20, 1000), group_size=256, bits=2, seed=0)


# ----------------------------------------------------------------- torch side
def draw_torch(spec: TensorSpec, device):
    """Materialise `spec` on `device` (flattened, contiguous)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(spec.data_seed)
    n = spec.numel
    if spec.law == SOFTMAX:
        z = torch.randn(n // spec.row, spec.row, device=device, generator=g,
                        dtype=torch.float32)
        z.mul_(2.0)
        x = torch.softmax(z, dim=-1).reshape(-1)
        del z
    else:
        x = torch.randn(n, device=device, generator=g, dtype=torch.float32)
        if spec.law == RELU:
            x.clamp_(min=0)
        elif spec.law == GELU:
            x = torch.nn.functional.gelu(x)
        elif spec.law == OUTLIER:
            k = max(n // 100, 1)
            pos = torch.randint(0, n, (k,), device=device, generator=g)
            x[pos] *= 10.0
        elif spec.law != NORMAL:
            raise ValueError(spec.law)
    if spec.dtype == "bf16":
        x = x.to(torch.bfloat16)
    return x.contiguous()


def lognormal_sensitivities(L: int, data_seed: int) -> np.ndarray:
    """c_l ~ LogNormal(0, 2) as float32."""
    rng = np.random.default_rng(data_seed)
    return rng.lognormal(mean=0.0, sigma=2.0, size=L).astype(np.float32)


# --------------------------------------------------------- activation sets
def resnet50_set(batch: int = 64) -> List[TensorSpec]:
    """The 53 convolution outputs of a ResNet-50-shaped net (bottleneck blocks,
    stride on the 3x3 convolution) at `batch` x 3 x 224 x 224.  Outputs that a
    ReLU follows are half zeros; third-conv and downsample outputs are N(0,1)."""
    specs: List[TensorSpec] = []

    def add(name, c, h, law):
        k = len(specs)
        specs.append(TensorSpec(name, (batch, c, h, h), law, "f32", 2000 + k, k))

    add("stem.conv", 64, 112, RELU)
    stages = [(64, 3, 56), (128, 4, 28), (256, 6, 14), (512, 3, 7)]
    h_in = 56
    for si, (w, blocks, h_out) in enumerate(stages):
        for b in range(blocks):
            h1 = h_in if b == 0 else h_out        # 1x1 conv runs before the stride
            add(f"s{si + 1}b{b}.conv1", w, h1, RELU)
            add(f"s{si + 1}b{b}.conv2", w, h_out, RELU)
            add(f"s{si + 1}b{b}.conv3", 4 * w, h_out, NORMAL)
            if b == 0:
                add(f"s{si + 1}b{b}.down", 4 * w, h_out, NORMAL)
        h_in = h_out
    return specs


def bert_large_set(batch: int = 32, seq: int = 512, hidden: int = 1024,
                   ffn: int = 4096, heads: int = 16, layers: int = 24) -> List[TensorSpec]:
    """Per layer: QKV input, softmax probabilities, GELU input, LayerNorm input."""
    specs: List[TensorSpec] = []
    for l in range(layers):
        for name, shape, law, row in (
            ("qkv_in", (batch, seq, hidden), NORMAL, 0),
            ("probs", (batch, heads, seq, seq), SOFTMAX, seq),
            ("gelu_in", (batch, seq, ffn), NORMAL, 0),
            ("ln_in", (batch, seq, hidden), NORMAL, 0),
        ):
            k = len(specs)
            specs.append(TensorSpec(f"l{l}.{name}", shape, law, "bf16", 3000 + k, k, row))
    return specs


def gcn_set(nodes: int = 169343, hidden: int = 256, layers: int = 3) -> List[TensorSpec]:
    return [TensorSpec(f"gcn{l}.relu", (nodes, hidden), RELU, "f32", 4000 + l, l)
            for l in range(layers)]


def vit_large_set(batch: int = 128, tokens: int = 197, hidden: int = 1024,
                  mlp: int = 4096, heads: int = 16, layers: int = 24) -> List[TensorSpec]:
    """400 tensors: 24 layers x 16 tensors (12 hidden-sized, 2 MLP-sized, 2
    attention-probability-sized) + 16 small extras."""
    specs: List[TensorSpec] = []

    def add(name, shape, law, row=0):
        k = len(specs)
        specs.append(TensorSpec(name, shape, law, "bf16", 5000 + k, k, row))

    for l in range(layers):
        for j in range(12):
            add(f"l{l}.h{j}", (batch, tokens, hidden), NORMAL)
        add(f"l{l}.gelu_in", (batch, tokens, mlp), NORMAL)
        add(f"l{l}.gelu_out", (batch, tokens, mlp), GELU)
        for j in range(2):
            add(f"l{l}.probs{j}", (batch, heads, tokens, tokens), SOFTMAX, tokens)
    for j in range(4):
        add(f"x.tok{j}", (batch, tokens, hidden), NORMAL)
    for j in range(4):
        add(f"x.patch{j}", (batch, tokens - 1, hidden), NORMAL)
    for j in range(4):
        add(f"x.cls{j}", (batch, hidden), NORMAL)
    for j in range(4):
        add(f"x.logit{j}", (batch, 1000), NORMAL)
    return specs
