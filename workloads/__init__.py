"""Seeded synthetic weight sets shaped like the paper's networks.

This module only draws random numbers and lays out shapes.  It holds none of
the compression arithmetic and is imported by tests and the benchmark to feed
the same host arrays to the CPU oracle and to the GPU library.

Stand-ins (the paper's trained checkpoints and datasets are not needed, the
compression step depends on shapes and value distribution only):

* ``single_matrix``     one 1024x1024 dense layer, N(0, 0.02^2)
* ``vgg19_cifar``       VGG-19 convolution stack of the CIFAR-10 experiment
                        (Evaluation, task 1; Table 2), Kaiming-normal
* ``resnet56_cifar``    ResNet-56 3x3 convolutions of the same experiment
* ``transformer_base``  6+6 layer Transformer-base matrices (the Introduction
                        motivates block-sparse Transformers), N(0, 0.02^2)
* ``lc_stress``         64 matrices of 4096x4608 with multipliers, the
                        large-model L-C step (Section 3.3)

Every tensor has its own PCG64 stream keyed by (seed, tensor index), so tensors
can be generated independently (and in parallel) and a sample of the tensors is
bit-identical to the same tensors inside the full set.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from typing import List, Sequence, Tuple

import numpy as np

Shape = Tuple[int, ...]


def normal_tensor(seed: int, index: int, shape: Shape, std: float) -> np.ndarray:
    """fp32 N(0, std^2) tensor from the stream keyed by (seed, index)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(index)])))
    n = int(np.prod(shape, dtype=np.int64)) if len(shape) else 1
    x = rng.standard_normal(n, dtype=np.float32)
    x *= np.float32(std)
    return x.reshape(shape)


def normal_tensors(seed: int, shapes: Sequence[Shape], stds: Sequence[float],
                   indices: Sequence[int] | None = None, threads: int = 8) -> List[np.ndarray]:
    """Generate several tensors (optionally a subset given by ``indices``)."""
    if indices is None:
        indices = range(len(shapes))
    jobs = [(seed, i, tuple(shapes[i]), float(stds[i])) for i in indices]
    if len(jobs) <= 1 or threads <= 1:
        return [normal_tensor(*j) for j in jobs]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda j: normal_tensor(*j), jobs))


def kaiming_std(shape: Shape) -> float:
    """std = sqrt(2 / fan_in), fan_in = product of all dims but the first."""
    fan_in = int(np.prod(shape[1:], dtype=np.int64))
    return math.sqrt(2.0 / fan_in)


# ---------------------------------------------------------------- shapes ----

def single_matrix_shapes() -> List[Shape]:
    return [(1024, 1024)]


def vgg19_cifar_shapes() -> List[Shape]:
    chans = [64, 64, 128, 128, 256, 256, 256, 256, 512, 512, 512, 512, 512, 512, 512, 512]
    shapes: List[Shape] = []
    cin = 3
    for c in chans:
        shapes.append((c, cin, 3, 3))
        cin = c
    shapes.append((10, 512))          # classifier, [out, in]
    return shapes


def resnet56_cifar_conv_shapes() -> List[Shape]:
    """55 3x3 convolutions: stem + 3 stages x 9 basic blocks x 2 convs."""
    shapes: List[Shape] = [(16, 3, 3, 3)]
    cin = 16
    for c in (16, 32, 64):
        for _ in range(18):
            shapes.append((c, cin, 3, 3))
            cin = c
    return shapes


def resnet56_cifar_linear_shape() -> Shape:
    return (10, 64)


def transformer_base_shapes(d_model: int = 512, ffn: int = 2048, n_enc: int = 6, n_dec: int = 6) -> List[Shape]:
    enc = [(d_model, d_model)] * 4 + [(ffn, d_model), (d_model, ffn)]
    dec = [(d_model, d_model)] * 8 + [(ffn, d_model), (d_model, ffn)]   # self + cross attention
    return enc * n_enc + dec * n_dec


def lc_stress_shapes(n_tensors: int = 64, rows: int = 4096, cols: int = 4608) -> List[Shape]:
    return [(rows, cols)] * n_tensors


# ---------------------------------------------------------------- recipes ---

SEED_SINGLE, SEED_VGG, SEED_RESNET, SEED_TRANSFORMER, SEED_LC_W, SEED_LC_LAMBDA = 1911, 2497, 56, 512, 4096, 4097


def single_matrix() -> List[np.ndarray]:
    sh = single_matrix_shapes()
    return normal_tensors(SEED_SINGLE, sh, [0.02] * len(sh))


def vgg19_cifar() -> List[np.ndarray]:
    sh = vgg19_cifar_shapes()
    return normal_tensors(SEED_VGG, sh, [kaiming_std(s) for s in sh])


def resnet56_cifar_convs() -> List[np.ndarray]:
    sh = resnet56_cifar_conv_shapes()
    return normal_tensors(SEED_RESNET, sh, [kaiming_std(s) for s in sh])


def transformer_base() -> List[np.ndarray]:
    sh = transformer_base_shapes()
    return normal_tensors(SEED_TRANSFORMER, sh, [0.02] * len(sh))


def lc_stress(indices: Sequence[int] | None = None, n_tensors: int = 64, rows: int = 4096,
              cols: int = 4608, threads: int = 8) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    """(w, lambda) tensor lists; w ~ N(0, 0.01^2), lambda ~ N(0, 1e-4) (variance)."""
    sh = lc_stress_shapes(n_tensors, rows, cols)
    w = normal_tensors(SEED_LC_W, sh, [0.01] * len(sh), indices, threads)
    lam = normal_tensors(SEED_LC_LAMBDA, sh, [0.01] * len(sh), indices, threads)
    return w, lam


LC_MU = 1e-3
LC_DENSITY = 0.1


def search_densities(n: int = 10, lo: float = 0.005, hi: float = 0.5) -> List[float]:
    """Geometric grid lo .. hi (n points), the candidate densities of one search."""
    if n == 1:
        return [lo]
    return [lo * (hi / lo) ** (j / (n - 1)) for j in range(n)]
