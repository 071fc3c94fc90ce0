"""Seeded synthetic workloads: tensor shapes and input values, nothing else.

This module holds none of the method's arithmetic.  It serves both the GPU tests/bench
and the CPU oracle's tests, and imports neither.  The paper trains ResNet/DenseNet/VGG
models on CIFAR and ImageNet (Sec. 4.1); only the *shapes* of the per-layer tensors
matter to the SESGD step, so every workload here is a list of per-tensor element counts
of a public architecture plus normally distributed values drawn from a seed.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np


# --------------------------------------------------------------------------- shapes
def tiny_sizes() -> List[int]:
    return [1000, 4096, 10]


def resnet20_sizes() -> List[int]:
    """CIFAR-style ResNet-20: stem 3x3 conv, 3 stages x 3 basic blocks (two 3x3 convs
    each) of width 16/32/64, a BatchNorm scale+shift after each conv, 64x10 FC + bias."""
    sizes = [3 * 16 * 9, 16, 16]
    c_in = 16
    for width in (16, 32, 64):
        for _block in range(3):
            for conv in range(2):
                ci = c_in if conv == 0 else width
                sizes += [ci * width * 9, width, width]
            c_in = width
    sizes += [64 * 10, 10]
    return sizes


def resnet50_sizes() -> List[int]:
    """ImageNet ResNet-50: 7x7 stem, stages of 3/4/6/3 bottleneck blocks (1x1, 3x3, 1x1,
    expansion 4), projection shortcut in the first block of each stage, BN after every
    conv, 2048x1000 FC + bias."""
    sizes = [7 * 7 * 3 * 64, 64, 64]
    c_in = 64
    for width, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            sizes += [c_in * width, width, width]
            sizes += [width * width * 9, width, width]
            sizes += [width * 4 * width, 4 * width, 4 * width]
            if b == 0:
                sizes += [c_in * 4 * width, 4 * width, 4 * width]
            c_in = 4 * width
    sizes += [2048 * 1000, 1000]
    return sizes


def resnet18_sizes() -> List[int]:
    """ImageNet ResNet-18: 7x7 stem, stages of 2/2/2/2 basic blocks (two 3x3 convs each) of
    width 64/128/256/512, a 1x1 projection shortcut in the first block of stages 2-4, BN after
    every conv, 512x1000 FC + bias."""
    sizes = [7 * 7 * 3 * 64, 64, 64]
    c_in = 64
    for width in (64, 128, 256, 512):
        for b in range(2):
            sizes += [c_in * width * 9, width, width]
            sizes += [width * width * 9, width, width]
            if b == 0 and c_in != width:
                sizes += [c_in * width, width, width]
            c_in = width
    sizes += [512 * 1000, 1000]
    return sizes


def densenet121_sizes() -> List[int]:
    """ImageNet DenseNet-121: 7x7 stem to 64 channels + BN, dense blocks of 6/12/24/16 layers
    (BN, 1x1 conv to 128, BN, 3x3 conv to 32 new channels), transitions (BN, 1x1 conv halving
    the channels) between them, a final BN, 1024x1000 classifier + bias."""
    sizes = [7 * 7 * 3 * 64, 64, 64]
    c = 64
    for bi, layers in enumerate((6, 12, 24, 16)):
        for _ in range(layers):
            sizes += [c, c, c * 128, 128, 128, 128 * 32 * 9]
            c += 32
        if bi < 3:
            sizes += [c, c, c * (c // 2)]
            c //= 2
    sizes += [c, c, c * 1000, 1000]
    return sizes


def vgg16_sizes() -> List[int]:
    """VGG-16: 13 3x3 convs with bias, then FC 25088x4096, 4096x4096, 4096x1000 with bias."""
    sizes = []
    c_in = 3
    for c_out in (64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512):
        sizes += [c_in * c_out * 9, c_out]
        c_in = c_out
    for fi, fo in ((25088, 4096), (4096, 4096), (4096, 1000)):
        sizes += [fi * fo, fo]
    return sizes


def bert_base_sizes() -> List[int]:
    """BERT-base: word/position/type embeddings + LayerNorm, 12 encoder layers of
    hidden 768 / FFN 3072, pooler."""
    h, ffn = 768, 3072
    sizes = [30522 * h, 512 * h, 2 * h, h, h]
    for _layer in range(12):
        for _proj in range(4):
            sizes += [h * h, h]
        sizes += [h, h]
        sizes += [h * ffn, ffn, ffn * h, h]
        sizes += [h, h]
    sizes += [h * h, h]
    return sizes


# --------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class Workload:
    name: str
    n: int                      # logical workers
    group_size: int             # workers per group (the paper's n/k)
    sizes: tuple                # elements per tensor, in parameter order
    param_std: float = 0.05
    grad_std: float = 1e-3
    lr: float = 0.1
    mu: float = 0.9
    iters: int = 10
    grad_dtype: str = "f32"     # "f32" or "bf16"

    @property
    def P(self) -> int:
        return int(sum(self.sizes))

    def layer_offsets(self, pitch: Optional[int] = None) -> np.ndarray:
        """Host int64 offsets; when pitch > P a final dummy layer carries the padding."""
        offs = [0]
        for s in self.sizes:
            offs.append(offs[-1] + int(s))
        if pitch is not None and pitch != offs[-1]:
            if pitch < offs[-1]:
                raise ValueError("pitch smaller than the model")
            offs.append(int(pitch))
        return np.asarray(offs, dtype=np.int64)

    @property
    def grad_bytes(self) -> int:
        return 2 if self.grad_dtype == "bf16" else 4


def _wl(name, n, m, sizes, **kw) -> Workload:
    return Workload(name=name, n=n, group_size=m, sizes=tuple(sizes), **kw)


WORKLOADS = {
    "tiny": _wl("tiny", 4, 2, tiny_sizes(), grad_std=1.0, mu=0.0, iters=5),
    "resnet20": _wl("resnet20", 16, 4, resnet20_sizes(), grad_std=1e-2, iters=100),
    "resnet50": _wl("resnet50", 16, 4, resnet50_sizes(), grad_std=1e-3, iters=50),
    "vgg16": _wl("vgg16", 32, 4, vgg16_sizes(), grad_std=1e-3, iters=20),
    # the other two networks of the paper's experiments (Sec. 4.1), at its 16 workers in 4 groups
    "resnet18": _wl("resnet18", 16, 4, resnet18_sizes(), grad_std=1e-3, iters=10),
    "densenet121": _wl("densenet121", 16, 4, densenet121_sizes(), grad_std=1e-3, iters=10),
    "bert_base": _wl("bert_base", 64, 8, bert_base_sizes(), grad_std=1e-3, lr=1e-4,
                     iters=10, grad_dtype="bf16"),
    "bert_base_full": _wl("bert_base_full", 64, 64, bert_base_sizes(), grad_std=1e-3,
                          lr=1e-4, iters=10, grad_dtype="bf16"),
}


# --------------------------------------------------------------------------- values
def _rng(*key_words) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(list(key_words))))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even) and return the uint16 patterns.
    Part of input generation: both the GPU path and the oracle consume these bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def host_params(n: int, ncols: int, std: float, seed: int = 0, pitch: Optional[int] = None
                ) -> np.ndarray:
    """One draw of ncols values, identical on every worker (all workers start from the
    same x_0, Sec. 3.2).  Padding columns, if any, are zero."""
    pitch = ncols if pitch is None else pitch
    out = np.zeros((n, pitch), np.float32)
    row = _rng(seed, 0x9A7A).standard_normal(ncols, dtype=np.float32) * np.float32(std)
    out[:, :ncols] = row[None, :]
    return out


def host_grads(n: int, ncols: int, std: float, seed: int, it: int, dtype: str = "f32",
               pitch: Optional[int] = None) -> np.ndarray:
    """Independent N(0, std) gradients per worker, fresh for iteration ``it``."""
    pitch = ncols if pitch is None else pitch
    out = np.zeros((n, pitch), np.float32)
    for i in range(n):
        out[i, :ncols] = _rng(seed, 0x6AAD, it, i).standard_normal(ncols, dtype=np.float32) \
            * np.float32(std)
    if dtype == "bf16":
        return f32_to_bf16_bits(out)
    return out


def sample_columns(pitch: int, count: int, seed: int = 0, tile: int = 1024) -> np.ndarray:
    """Sorted column sample for full-size spot checks: the first and last ``tile`` columns,
    a run straddling a tile boundary in the middle, and uniformly random columns."""
    if pitch <= 4 * tile:
        return np.arange(pitch, dtype=np.int64)
    mid = (pitch // 2 // tile) * tile
    fixed = np.concatenate([np.arange(0, tile), np.arange(mid - tile // 2, mid + tile // 2),
                            np.arange(pitch - tile, pitch)])
    rnd = _rng(seed, 0x5A3B).integers(0, pitch, size=max(count - fixed.size, 0))
    return np.unique(np.concatenate([fixed, rnd]).astype(np.int64))


def stratified_columns(pitch: int, whole_tiles: int, random_count: int, seed: int = 0,
                       tile: int = 256) -> np.ndarray:
    """Sorted column sample made of whole tiles of ``tile`` columns (the first, the last, and
    evenly spaced ones in between: ``whole_tiles`` in all) plus ``random_count`` uniformly random
    columns.  256 fp32 columns are the 1 KiB piece of a row that one wavefront moves per access."""
    ntiles = (pitch + tile - 1) // tile
    if ntiles <= whole_tiles:
        return np.arange(pitch, dtype=np.int64)
    picks = np.unique(np.linspace(0, ntiles - 1, whole_tiles).astype(np.int64))
    cols = (picks[:, None] * tile + np.arange(tile)[None, :]).reshape(-1)
    cols = cols[cols < pitch]
    rnd = _rng(seed, 0x57A7).integers(0, pitch, size=random_count)
    return np.unique(np.concatenate([cols, rnd]).astype(np.int64))
