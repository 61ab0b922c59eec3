"""Synthetic workloads: tensor shape lists and seeded gradient generators.

This module holds no PowerSGD arithmetic.  It only says which tensors a model
has (shapes from the paper's Appendix F tables, "Parameters in the ResNet18
architecture" and "Parameters in the LSTM architecture", and the transformer
language model of Appendix D) and draws seeded synthetic gradients of those
shapes.  Both the GPU tests/benchmark and the CPU oracle's tests take their
inputs from here; neither side's arithmetic lives here.

Gradient recipe (stand-in for the CIFAR10 / WikiText gradients, which are not
available): for matrix i, step t, worker w

    G = U diag(s) V^T + sigma * Z

U (n x k'), V (m x k') orthonormal from the QR of seeded Gaussian matrices
(columns sign-fixed so that diag(R) > 0), drawn once per matrix and shared by
all workers and steps; k' = min(k, n, m); Z iid N(0,1) redrawn for every
(step, worker).  sigma is a standard deviation.  1-D tensors are iid
N(0, sigma^2).  An optional row mask (fresh uniform subset of rows per step)
zeroes all other rows of G, planted term and noise alike, to imitate a sparse
embedding gradient.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np


@dataclass
class Workload:
    name: str
    shapes: List[Tuple[int, ...]]            # 2-D (n, m) matrices and 1-D (L,) vectors, model order
    planted_rank: int
    singular_values: np.ndarray              # length planted_rank
    sigma: float                             # noise std
    row_density: dict = field(default_factory=dict)   # tensor index -> fraction of nonzero rows
    grad_dtype: str = "f32"                  # "f32" or "bf16"

    @property
    def matrix_indices(self):
        return [i for i, s in enumerate(self.shapes) if len(s) >= 2]

    @property
    def vector_indices(self):
        return [i for i, s in enumerate(self.shapes) if len(s) == 1]

    @property
    def n_matrix_elems(self):
        return int(sum(int(np.prod(self.shapes[i])) for i in self.matrix_indices))

    @property
    def n_vector_elems(self):
        return int(sum(self.shapes[i][0] for i in self.vector_indices))


# --------------------------------------------------------------------------
# shape lists
# --------------------------------------------------------------------------

def tiny_shapes():
    return [(64, 27)] + [(64, 576)] * 4


def resnet18_shapes(with_vectors=True):
    """ResNet18 for CIFAR10 as in the paper's Appendix F table: conv kernels
    o x i x k x k seen as o x (i k k), shortcut 1x1 convs, the 10 x 512
    classifier, and (optionally) the batch-norm / bias vectors, 9 610 values
    in total (the table's 38 KB of 'Bias vectors')."""
    shapes: List[Tuple[int, ...]] = []

    def bn(c):
        if with_vectors:
            shapes.append((c,))
            shapes.append((c,))

    shapes.append((64, 27)); bn(64)                       # conv1
    for _ in range(2):                                     # layer1: 2 blocks
        shapes.append((64, 576)); bn(64)
        shapes.append((64, 576)); bn(64)
    for stage_in, c in ((64, 128), (128, 256), (256, 512)):  # layer2..4
        shapes.append((c, stage_in * 9)); bn(c)            # block0.conv1
        shapes.append((c, c * 9)); bn(c)                   # block0.conv2
        shapes.append((c, stage_in)); bn(c)                # block0.shortcut (1x1)
        shapes.append((c, c * 9)); bn(c)                   # block1.conv1
        shapes.append((c, c * 9)); bn(c)                   # block1.conv2
    shapes.append((10, 512))                               # linear
    if with_vectors:
        shapes.append((10,))
    return shapes


def lstm_shapes(vocab=33280, with_vectors=True):
    """3-layer LSTM language model, hidden 650 (Appendix F): tied
    encoder/decoder vocab x 650, per layer W_ih and W_hh of 2600 x 650, and
    the bias vectors (two of 2600 per layer, one of vocab for the decoder)."""
    shapes: List[Tuple[int, ...]] = [(vocab, 650)]
    for _ in range(3):
        shapes.append((2600, 650))
        shapes.append((2600, 650))
        if with_vectors:
            shapes.append((2600,))
            shapes.append((2600,))
    if with_vectors:
        shapes.append((vocab,))
    return shapes


def transformer_shapes(layers=24, d=2048, ff=8192, vocab=50304, with_vectors=True):
    """Transformer language model shaped like Appendix D's setting: per layer
    four d x d attention projections, ff x d and d x ff feed-forward
    matrices; one vocab x d embedding.  Vectors (a choice of this build): per
    layer two layer norms (weight + bias), four projection biases, two
    feed-forward biases; one final layer norm."""
    shapes: List[Tuple[int, ...]] = [(vocab, d)]
    for _ in range(layers):
        for _ in range(4):
            shapes.append((d, d))
            if with_vectors:
                shapes.append((d,))
        shapes.append((ff, d))
        if with_vectors:
            shapes.append((ff,))
        shapes.append((d, ff))
        if with_vectors:
            shapes.append((d,))
        if with_vectors:
            shapes.extend([(d,)] * 4)
    if with_vectors:
        shapes.extend([(d,)] * 2)
    return shapes


def tiny(seed=0):
    return Workload("tiny", tiny_shapes(), 4, np.array([1.0, 0.5, 0.25, 0.125]), 0.01)


def resnet18():
    return Workload("resnet18", resnet18_shapes(), 8, 1.0 / np.arange(1, 9), 0.01)


def lstm():
    wl = Workload("lstm", lstm_shapes(), 16, 1.0 / np.arange(1, 17), 0.01)
    wl.row_density = {0: 0.05}
    return wl


def transformer(layers=24):
    return Workload("transformer%d" % layers, transformer_shapes(layers=layers), 64,
                    1.0 / np.arange(1, 65), 0.001, grad_dtype="bf16")


def by_name(name: str) -> Workload:
    table = {"tiny": tiny, "resnet18": resnet18, "lstm": lstm, "transformer": transformer}
    return table[name]()


# --------------------------------------------------------------------------
# numpy generators (host; used for parity runs)
# --------------------------------------------------------------------------

def _rng(*key):
    return np.random.default_rng(np.random.SeedSequence([int(k) for k in key]))


def _orthonormal(rng, n, k):
    a = rng.standard_normal((n, k))
    q, r = np.linalg.qr(a)
    sgn = np.sign(np.diag(r))
    sgn[sgn == 0] = 1.0
    return q * sgn[None, :]


def planted_factors(wl: Workload, seed: int, only=None):
    """Per matrix tensor: (U*s, V) with k' = min(k, n, m) columns; None for vectors (and, when `only`
    is a collection of tensor indices, for every tensor outside it: each tensor has its own seeded stream,
    so a subset is generated exactly as it would be within the whole set)."""
    out = []
    for i, s in enumerate(wl.shapes):
        if len(s) < 2 or (only is not None and i not in only):
            out.append(None)
            continue
        n, m = s
        k = min(wl.planted_rank, n, m)
        rng = _rng(seed, 1000003, i)
        U = _orthonormal(rng, n, k)
        V = _orthonormal(rng, m, k)
        out.append((U * wl.singular_values[:k][None, :], V))
    return out


def gradients(wl: Workload, factors, seed: int, step: int, worker: int, only=None):
    """List of float32 arrays (one per tensor) for (step, worker); None outside `only` when it is given."""
    out = []
    for i, s in enumerate(wl.shapes):
        if only is not None and i not in only:
            out.append(None)
            continue
        rng = _rng(seed, i, step, worker)
        if len(s) < 2:
            out.append((wl.sigma * rng.standard_normal(s)).astype(np.float32))
            continue
        Us, V = factors[i]
        g = Us @ V.T + wl.sigma * rng.standard_normal(s)
        dens = wl.row_density.get(i)
        if dens is not None:
            # the row subset depends on the step only: same rows on every worker
            mrng = _rng(seed, 2000003, i, step)
            keep = mrng.random(s[0]) < dens
            g = g * keep[:, None]
        out.append(g.astype(np.float32))
    return out


def initial_q(wl: Workload, rank: int, seed: int, only=None):
    """Q0 iid N(0,1) per matrix (m x min(r, n, m)), float32; None for vectors (and outside `only`)."""
    out = []
    for i, s in enumerate(wl.shapes):
        if len(s) < 2 or (only is not None and i not in only):
            out.append(None)
            continue
        n, m = s
        r = min(rank, n, m)
        out.append(_rng(seed, 3000003, i).standard_normal((m, r)).astype(np.float32))
    return out


def kept_count(shape, rank: int) -> int:
    """Entries per matrix that the Random Block / Random K baselines keep: (n + m) r, at most n m."""
    n, m = shape
    return min((n + m) * rank, n * m)


def block_starts(wl: Workload, rank: int, seed: int, step: int):
    """The draw of the Random Block baseline: per matrix one start index uniform in [0, n m), the same on every
    worker (it depends on the seed and the step only); None for vectors."""
    out = []
    for i, s in enumerate(wl.shapes):
        if len(s) < 2:
            out.append(None)
            continue
        out.append(int(_rng(seed, 4000003, i, step).integers(0, s[0] * s[1])))
    return out


def random_indices(wl: Workload, rank: int, seed: int, step: int):
    """The draw of the Random K baseline: per matrix kept_count positions in [0, n m) without repetition, the same
    on every worker; int64 arrays, None for vectors."""
    out = []
    for i, s in enumerate(wl.shapes):
        if len(s) < 2:
            out.append(None)
            continue
        out.append(_rng(seed, 5000003, i, step).choice(s[0] * s[1], size=kept_count(s, rank), replace=False)
                   .astype(np.int64))
    return out


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even), returned as
    float32 holding exactly representable values.  Input conditioning for the
    bf16-gradient workload, not part of the method."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    rounded = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16_round(a)."""
    r = bf16_round(a)
    return (r.view(np.uint32) >> 16).astype(np.uint16)
