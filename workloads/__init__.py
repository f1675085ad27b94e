"""Seeded synthetic inputs for the CD-GraB pair-balancing path.

This package only *produces inputs* (gradient rows, softmax-regression problems,
workload shape tables).  It holds none of the method's arithmetic -- no
balancing, no reordering, no gradient formula -- so both the CPU oracle's tests
and the HIP library's tests may draw their inputs from it.

Two families:
  * numpy generators for the small configurations (everything below), and
  * the counter-based streaming generator for the large ones
    (``workloads.synth``: one C header compiled for the host and for gfx950,
    bit-identical on both).

The five workload shapes stand in for the paper's tasks (none of its datasets is
available): a unit-test-sized epoch, a 784->10 softmax regression (the paper's
own convex task is an 18-feature logistic regression), an LSTM-sized vector with
32 workers, a ResNet-18-sized vector and a GPT-2-small-sized vector.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    m: int            # simulated workers
    n: int            # examples per worker (even)
    d: int            # parameters
    kind: str         # "dense" (rows materialised), "softmax", "stream" (generator)
    block_scales: int = 0      # number of contiguous scale blocks along d (0 = none)
    zero_fraction: float = 0.0  # per-row Bernoulli probability of an exact zero


CONFIGS = {
    "c1_tiny": Workload("c1_tiny", m=4, n=64, d=1024, kind="dense"),
    "c2_softmax": Workload("c2_softmax", m=16, n=3750, d=7850, kind="softmax"),
    "c3_stream_1m": Workload("c3_stream_1m", m=32, n=1024, d=1 << 20, kind="stream"),
    "c4_resnet18": Workload("c4_resnet18", m=32, n=512, d=11_200_000, kind="stream",
                            block_scales=64),
    "c5_gpt2s": Workload("c5_gpt2s", m=8, n=256, d=124_000_000, kind="stream",
                         zero_fraction=0.2),
}


def tiny_epoch(seed: int, m: int = 4, n: int = 64, d: int = 1024) -> np.ndarray:
    """Rows z[m][n][d] fp32: a shared mean 0.1*N(0,1)^d plus N(0,1)^d per row."""
    rng = np.random.default_rng(seed)
    mu = 0.1 * rng.standard_normal(d)
    z = mu[None, None, :] + rng.standard_normal((m, n, d))
    return z.astype(np.float32)


def integer_rows(seed: int, m: int, n: int, d: int, maxabs: int = 8) -> np.ndarray:
    """Rows with small integer values: every fp32/fp64 sum and product the path
    forms on them is exact, so any two correct implementations agree bit for bit,
    ties included (many pair dots are exactly zero)."""
    rng = np.random.default_rng(seed)
    return rng.integers(-maxabs, maxabs + 1, size=(m, n, d)).astype(np.float32)


def heavy_rows(seed: int, m: int, n: int, d: int) -> np.ndarray:
    """Rows shaped like the streaming configs but drawn with numpy: shared mean
    0.1*N(0,1) plus Student-t(3) noise times a per-row log-normal(0.5) scale."""
    rng = np.random.default_rng(seed)
    mu = 0.1 * rng.standard_normal(d)
    scale = np.exp(0.5 * rng.standard_normal((m, n, 1)))
    z = mu[None, None, :] + scale * rng.standard_t(3.0, size=(m, n, d))
    return z.astype(np.float32)


def softmax_problem(seed: int, N: int, in_dim: int = 784, classes: int = 10):
    """X[N][in_dim] ~ U[0,1) fp32, y[N] ~ U{0..classes-1} int32,
    W[(in_dim+1)][classes] ~ N(0, sigma=0.01) fp32 (last row is the bias)."""
    rng = np.random.default_rng(seed)
    X = rng.random((N, in_dim), dtype=np.float32)
    y = rng.integers(0, classes, size=N).astype(np.int32)
    W = (0.01 * rng.standard_normal((in_dim + 1, classes))).astype(np.float32)
    return X, y, W


def random_perms(seed: int, m: int, n: int) -> np.ndarray:
    """m independent uniformly random permutations of range(n), int32."""
    rng = np.random.default_rng(seed)
    return np.stack([rng.permutation(n) for _ in range(m)]).astype(np.int32)


def random_signs(seed: int, m: int, n: int) -> np.ndarray:
    """Per-example +-1 signs [m][n], int8."""
    rng = np.random.default_rng(seed)
    return (2 * rng.integers(0, 2, size=(m, n)) - 1).astype(np.int8)


def herding_vectors(seed: int, N: int, d: int = 16) -> np.ndarray:
    """The vectors of the paper's synthetic herding-bound study (App. E): N draws
    from Unif(0,1)^d, zero-centred over the set, each scaled to unit L2 norm."""
    rng = np.random.default_rng(seed)
    z = rng.random((N, d))
    z -= z.mean(axis=0, keepdims=True)
    z /= np.linalg.norm(z, axis=1, keepdims=True)
    return z.astype(np.float32)
