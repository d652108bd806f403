"""Seeded synthetic inputs for the NOVAK update step: tensor-shape lists and value generators.

This module holds NO optimizer arithmetic.  It is the only code that the CPU oracle's tests and the
HIP path's tests/bench both use: it builds the parameter-shape lists of the five benchmark
workloads and draws parameters / gradients from seeded generators so that both sides see the same
bits.  The shapes stand in for the paper's ImageNet / CIFAR training runs (section 9 of the paper);
only shapes and value scales matter to the per-parameter update.

Value recipe ("N(0, s)" is read as mean 0, standard deviation s):
  parameters  ~ N(0, 0.02)
  gradients   ~ N(0, grad_std), a fresh draw per step, optionally rounded to bf16 (round-to-nearest-even)
  m = v = 0 at t = 0.
Seeds 42, 100, 2025 are the three seeds the paper's experiments use (section 9.1).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

PAPER_SEEDS = (42, 100, 2025)
PARAM_STD = 0.02

Shape = Tuple[int, ...]


def _numel(shape: Shape) -> int:
    return int(math.prod(shape))


# ----------------------------------------------------------------------------------------------
# shape lists
# ----------------------------------------------------------------------------------------------
def flat_shapes(n: int = 1 << 20) -> List[Shape]:
    """One flat tensor of n elements (2^20 by default)."""
    return [(n,)]


def resnet50_shapes() -> List[Shape]:
    """ResNet-50: 7x7 stem, stages [3,4,6,3] of 1x1/3x3/1x1 bottlenecks, BN pairs, fc 1000x2048."""
    out: List[Shape] = []

    def conv_bn(cout: int, cin: int, k: int) -> None:
        out.append((cout, cin, k, k))
        out.append((cout,))  # BN gamma
        out.append((cout,))  # BN beta

    conv_bn(64, 3, 7)
    cin = 64
    for width, blocks in zip((64, 128, 256, 512), (3, 4, 6, 3)):
        for b in range(blocks):
            conv_bn(width, cin, 1)
            conv_bn(width, width, 3)
            conv_bn(4 * width, width, 1)
            if b == 0:
                conv_bn(4 * width, cin, 1)  # downsample branch
            cin = 4 * width
    out.append((1000, 2048))
    out.append((1000,))
    return out


def vgg16_shapes() -> List[Shape]:
    """VGG-16: 13 conv3x3 (+bias) and three fully connected layers (+bias)."""
    out: List[Shape] = []
    cin = 3
    for cout in (64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512):
        out.append((cout, cin, 3, 3))
        out.append((cout,))
        cin = cout
    for o, i in ((4096, 25088), (4096, 4096), (1000, 4096)):
        out.append((o, i))
        out.append((o,))
    return out


def vit_b16_shapes() -> List[Shape]:
    """ViT-B/16: patch embedding, cls/pos tokens, 12 encoder blocks, final LayerNorm, head."""
    d, mlp = 768, 3072
    out: List[Shape] = [(d, 3, 16, 16), (d,), (1, 1, d), (1, 197, d)]
    for _ in range(12):
        out += [(d,), (d,)]                      # LayerNorm 1
        out += [(3 * d, d), (3 * d,)]            # qkv
        out += [(d, d), (d,)]                    # attention projection
        out += [(d,), (d,)]                      # LayerNorm 2
        out += [(mlp, d), (mlp,)]                # MLP up
        out += [(d, mlp), (d,)]                  # MLP down
    out += [(d,), (d,)]                          # final LayerNorm
    out += [(1000, d), (1000,)]                  # classification head
    return out


def decoder_1p3b_shapes() -> List[Shape]:
    """1.3B decoder: vocab 50257 embedding, 2048 learned positions, 24 blocks of d=2048 / mlp 8192."""
    d, mlp, vocab, ctx = 2048, 8192, 50257, 2048
    out: List[Shape] = [(vocab, d), (ctx, d)]
    for _ in range(24):
        out += [(d,), (d,)]
        out += [(3 * d, d), (3 * d,)]
        out += [(d, d), (d,)]
        out += [(d,), (d,)]
        out += [(mlp, d), (mlp,)]
        out += [(d, mlp), (d,)]
    out += [(d,), (d,)]
    return out


def ragged_shapes() -> List[Shape]:
    """Odd sizes that exercise tails, one-element tensors and chunk boundaries (not a paper workload)."""
    return [(1,), (3,), (7,), (64,), (255,), (1021,), (4096,), (4099,), (16384 + 5,), (65536 + 1,),
            (3, 5, 7), (2, 65536 + 3), (300007,)]


@dataclass(frozen=True)
class Workload:
    """A named benchmark configuration: shapes, value scales and the hyper-parameters it is run with."""
    name: str
    shapes: Tuple[Shape, ...]
    grad_std: float
    grad_dtype: str              # "f32" or "bf16"
    steps: int
    hyper: Dict[str, object] = field(default_factory=dict)

    @property
    def numels(self) -> List[int]:
        return [_numel(s) for s in self.shapes]

    @property
    def total(self) -> int:
        return sum(self.numels)

    @property
    def rows(self) -> List[int]:
        """Size of the first dimension of tensors with more than one dimension, else 0."""
        return [int(s[0]) if len(s) > 1 else 0 for s in self.shapes]


# Hyper-parameters shared by every configuration unless a workload overrides them.
BASE_HYPER: Dict[str, object] = dict(
    lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=1e-2, beta_n=0.9,
    la_alpha=0.5, la_k=5, rectified=True, decoupled_decay=True,
    nesterov="approx", lookahead="memory_efficient", unrect_fallback="adam_denom", mode="fast",
)


def _wl(name, shapes, grad_std, grad_dtype, steps, **over) -> Workload:
    h = dict(BASE_HYPER)
    h.update(over)
    return Workload(name, tuple(shapes), grad_std, grad_dtype, steps, h)


def get_workload(name: str) -> Workload:
    """The five benchmark configurations (C1..C5) and the ragged edge-case list."""
    if name == "c1_flat_1m":
        return _wl(name, flat_shapes(), 1e-2, "f32", 100, mode="research")
    if name == "c2_resnet50":
        return _wl(name, resnet50_shapes(), 1e-3, "f32", 10)
    if name == "c3_vgg16":
        return _wl(name, vgg16_shapes(), 1e-3, "f32", 10)
    if name == "c4_vit_b16_bf16":
        return _wl(name, vit_b16_shapes(), 1e-3, "bf16", 100)
    if name == "c5_decoder_1p3b":
        return _wl(name, decoder_1p3b_shapes(), 1e-3, "f32", 11)
    if name == "ragged":
        return _wl(name, ragged_shapes(), 1e-2, "f32", 11, mode="research")
    raise KeyError(name)


WORKLOAD_NAMES = ("c1_flat_1m", "c2_resnet50", "c3_vgg16", "c4_vit_b16_bf16", "c5_decoder_1p3b")


# ----------------------------------------------------------------------------------------------
# value generators (host side, numpy)
# ----------------------------------------------------------------------------------------------
def _rng(seed: int, role: str, tensor: int, step: int = 0) -> np.random.Generator:
    """One independent Philox stream per (seed, role, tensor index, step)."""
    role_id = {"param": 1, "grad": 2}[role]
    return np.random.Generator(np.random.Philox(key=[(seed << 8) | role_id, (tensor << 32) | step]))


def host_params(numels: Sequence[int], seed: int = 42) -> List[np.ndarray]:
    """fp32 parameter tensors ~ N(0, 0.02), flattened."""
    return [(_rng(seed, "param", i).standard_normal(n, dtype=np.float32) * np.float32(PARAM_STD))
            for i, n in enumerate(numels)]


def host_grads(numels: Sequence[int], step: int, grad_std: float, seed: int = 42,
               bf16: bool = False) -> List[np.ndarray]:
    """fp32 gradient tensors ~ N(0, grad_std) for 1-based `step`.

    With bf16=True each value is rounded to the nearest bfloat16 (ties to even) and returned as the
    fp32 number with that exact value, so every consumer sees identical gradient values.
    """
    out = []
    for i, n in enumerate(numels):
        g = _rng(seed, "grad", i, step).standard_normal(n, dtype=np.float32) * np.float32(grad_std)
        out.append(round_to_bf16(g) if bf16 else g)
    return out


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); result kept in fp32 storage."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    nan = np.isnan(x)
    res = r.astype(np.uint32).view(np.float32).copy()
    res[nan] = np.nan
    return res


def bf16_bits(x_rounded: np.ndarray) -> np.ndarray:
    """The 16-bit patterns of values that are already exactly representable in bfloat16."""
    return (np.ascontiguousarray(x_rounded, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def sample_indices(numel: int, n_samples: int, seed: int, tensor: int, block: int = 0) -> np.ndarray:
    """Sorted unique element indices used for sampled parity at full workload sizes.

    Always contains the first and last 16 elements; if `block` is given it also contains the four
    elements on either side of every multiple of `block` for a few randomly chosen multiples, so
    that chunk boundaries of the multi-tensor table are covered.
    """
    rng = np.random.Generator(np.random.Philox(key=[seed, (tensor << 8) | 0xA5]))
    idx = [np.arange(min(16, numel)), np.arange(max(0, numel - 16), numel)]
    if numel > 32:
        idx.append(rng.integers(0, numel, size=min(n_samples, numel), dtype=np.int64))
    if block and numel > block:
        nb = numel // block
        which = rng.integers(1, nb + 1, size=min(8, nb), dtype=np.int64) * block
        for w in which:
            idx.append(np.arange(max(0, w - 4), min(numel, w + 4)))
    return np.unique(np.concatenate(idx).astype(np.int64))
