"""Seeded synthetic workloads: model-shaped tensor lists and input generators.

This module holds none of the method's arithmetic.  It only says how large the
parameter tensors of the paper's models are (App. B, workloads: GPT-Neo with 8M
and 125M parameters, ResNet-50 with 25.6M parameters, the small CNN of the
CIFAR-10 simulation table) and draws seeded initial models, quadratic targets
and noisy gradients.  It serves the device path's tests and benchmark and the
CPU checker alike; neither of those imports the other.

The paper's datasets and trained weights are not needed by the update path: its
cost and its arithmetic depend on tensor sizes only, so seeded random tensors
of the models' shapes stand in for them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

PAD = 64    # every tensor starts at a multiple of 64 elements inside a flat row
ROW = 256   # the padded row length is a multiple of 256 elements


def _prod(shape: Sequence[int]) -> int:
    return int(math.prod(shape))


def gpt_neo_tensors(d: int, layers: int, vocab: int, positions: int) -> List[Tuple[str, Tuple[int, ...]]]:
    """GPT-Neo parameter tensors for hidden size d (App. B: 125M = d 768, 12 layers,
    1024 positions; vocabulary 50257 as in the public GPT-Neo configuration)."""
    t: List[Tuple[str, Tuple[int, ...]]] = [("wte", (vocab, d)), ("wpe", (positions, d))]
    for i in range(layers):
        p = f"h{i}."
        t += [(p + "ln1.w", (d,)), (p + "ln1.b", (d,)),
              (p + "attn.q", (d, d)), (p + "attn.k", (d, d)), (p + "attn.v", (d, d)),
              (p + "attn.o", (d, d)), (p + "attn.o.b", (d,)),
              (p + "ln2.w", (d,)), (p + "ln2.b", (d,)),
              (p + "mlp.fc.w", (4 * d, d)), (p + "mlp.fc.b", (4 * d,)),
              (p + "mlp.proj.w", (d, 4 * d)), (p + "mlp.proj.b", (d,))]
    t += [("ln_f.w", (d,)), ("ln_f.b", (d,))]
    return t


def gpt_neo_8m_like_tensors() -> List[Tuple[str, Tuple[int, ...]]]:
    """Eight stacked tensors with GPT-Neo-8M's sizes (App. B: d 128, 8 layers, 300 positions):
    token and position embeddings, the 8 layers' attention / fc / proj matrices stacked, and
    three small groups for biases and norms.  2^23 = 8,388,608 parameters in total."""
    return [("wte", (50257, 128)), ("wpe", (300, 128)),
            ("attn_stack", (8, 4, 128, 128)), ("fc_stack", (8, 512, 128)), ("proj_stack", (8, 128, 512)),
            ("bias_stack", (10240,)), ("ln_f", (256,)), ("rest", (333952,))]


def resnet50_tensors() -> List[Tuple[str, Tuple[int, ...]]]:
    """ResNet-50 parameter tensors (App. B: the standard 50-layer bottleneck network, 1000 classes)."""
    t: List[Tuple[str, Tuple[int, ...]]] = [("conv1", (64, 3, 7, 7)), ("bn1.w", (64,)), ("bn1.b", (64,))]
    inplanes = 64
    for li, (planes, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for b in range(blocks):
            p = f"layer{li + 1}.{b}."
            t += [(p + "conv1", (planes, inplanes, 1, 1)), (p + "bn1.w", (planes,)), (p + "bn1.b", (planes,)),
                  (p + "conv2", (planes, planes, 3, 3)), (p + "bn2.w", (planes,)), (p + "bn2.b", (planes,)),
                  (p + "conv3", (planes * 4, planes, 1, 1)), (p + "bn3.w", (planes * 4,)), (p + "bn3.b", (planes * 4,))]
            if b == 0:
                t += [(p + "down.conv", (planes * 4, inplanes, 1, 1)),
                      (p + "down.bn.w", (planes * 4,)), (p + "down.bn.b", (planes * 4,))]
            inplanes = planes * 4
    t += [("fc.w", (1000, 2048)), ("fc.b", (1000,))]
    return t


def small_cnn_tensors() -> List[Tuple[str, Tuple[int, ...]]]:
    """The small CNN of the CIFAR-10 simulation study (App. B, architecture table)."""
    return [("conv1.w", (32, 3, 5, 5)), ("conv1.b", (32,)), ("conv2.w", (64, 32, 5, 5)), ("conv2.b", (64,)),
            ("fc1.w", (1024, 64 * 8 * 8)), ("fc1.b", (1024,)), ("fc2.w", (10, 1024)), ("fc2.b", (10,))]


@dataclass
class Workload:
    """One benchmark / parity configuration: sizes and hyper-parameters."""
    name: str
    K: int
    tensors: List[Tuple[str, Tuple[int, ...]]]
    inner: str = "adamw"            # "adamw" | "sgdm"
    grad_dtype: str = "f32"         # "f32" | "bf16"
    alpha: float = 1e-3             # inner learning rate (App. B: 0.001 for GPT-Neo and ResNet-50)
    eta: float = 16.0               # mixing rate (App. B: eta_t = 16 for GPT-Neo)
    p: float = 0.1
    H: int = 16
    steps: int = 64
    sigma: float = 0.01             # std of the gradient noise
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    momentum: float = 0.9
    outer_lr: float = 0.2           # App. B: outer learning rate 0.1 to 0.2
    outer_momentum: float = 0.9
    outer_nesterov: bool = True
    seed: int = 0
    extra: Dict[str, object] = field(default_factory=dict)

    @property
    def numels(self) -> List[int]:
        return [_prod(s) for _, s in self.tensors]

    @property
    def P(self) -> int:
        return sum(self.numels)


def workload(name: str) -> Workload:
    """The five configurations the benchmark and parity suites use."""
    if name == "gptneo8m_k4":
        return Workload(name, 4, gpt_neo_8m_like_tensors(), "adamw", "f32", p=0.1, H=16, steps=64, sigma=0.01, seed=0)
    if name == "gptneo125m_k8":
        return Workload(name, 8, gpt_neo_tensors(768, 12, 50257, 1024), "adamw", "bf16", p=0.05, H=64, steps=256,
                        sigma=0.1, seed=1)
    if name == "resnet50_k8":
        return Workload(name, 8, resnet50_tensors(), "sgdm", "f32", p=0.1, H=32, steps=64, sigma=0.01,
                        weight_decay=1e-4, momentum=0.9, seed=2)
    if name == "gptneo125m_k16":
        return Workload(name, 16, gpt_neo_tensors(768, 12, 50257, 1024), "adamw", "f32", p=0.02, H=128, steps=256,
                        sigma=0.1, outer_lr=0.7, outer_momentum=0.9, seed=3)
    if name == "gptneo1p3b_k8":
        return Workload(name, 8, gpt_neo_tensors(2048, 24, 50257, 2048), "adamw", "bf16", p=0.05, H=64, steps=128,
                        sigma=0.1, seed=4)
    if name == "smallcnn_k64":
        return Workload(name, 64, small_cnn_tensors(), "sgdm", "f32", p=0.25, H=32, steps=64, eta=1.0,
                        weight_decay=0.0, outer_lr=0.1, seed=5)
    raise KeyError(name)


WORKLOADS = ("gptneo8m_k4", "gptneo125m_k8", "resnet50_k8", "gptneo125m_k16", "gptneo1p3b_k8", "smallcnn_k64")


def flat_layout(numels: Sequence[int]) -> Tuple[List[int], int]:
    """Start element of every tensor inside a flat row (each start rounded up to a
    multiple of PAD) and the padded row length (a multiple of ROW)."""
    offs, cur = [], 0
    for n in numels:
        offs.append(cur)
        cur = (cur + int(n) + PAD - 1) // PAD * PAD
    return offs, (cur + ROW - 1) // ROW * ROW


def real_mask(numels: Sequence[int]) -> np.ndarray:
    """Boolean row mask: True on tensor elements, False on padding."""
    offs, row = flat_layout(numels)
    m = np.zeros(row, bool)
    for o, n in zip(offs, numels):
        m[o:o + n] = True
    return m


def host_inputs(numels: Sequence[int], seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Initial model x0 ~ 0.02 N(0,1) and quadratic target c ~ N(0,1) as padded fp32
    rows (padding zero), from a seeded numpy generator."""
    rng = np.random.default_rng(seed)
    mask = real_mask(numels)
    x0 = (0.02 * rng.standard_normal(mask.size, dtype=np.float32)).astype(np.float32)
    c = rng.standard_normal(mask.size, dtype=np.float32)
    x0[~mask] = 0.0
    c[~mask] = 0.0
    return x0, c


def host_gradients(X: np.ndarray, c: np.ndarray, sigma: float, mask: np.ndarray,
                   rng: np.random.Generator) -> np.ndarray:
    """Synthetic stochastic gradients of f(x) = 0.5 |x - c|^2 with additive noise,
    g_k = (x_k - c) + sigma N(0,1), for all K rows of X; fp32, zero on padding."""
    g = (X - c[None, :]) + np.float32(sigma) * rng.standard_normal(X.shape, dtype=np.float32)
    g = g.astype(np.float32)
    g[:, ~mask] = 0.0
    return g


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> bf16 bit patterns (uint16), round to nearest even."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32 values (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
