"""Seeded synthetic workloads: shapes and input generators only.

This module holds none of the method's arithmetic.  It names the shapes
(m, n, k, s, p, batch) that are measured and tested, and draws the input
vectors and kernels for them with numpy's default_rng, so that the GPU path
and whatever it is compared with receive the very same host arrays.

The paper's experiment (Section 4.1) draws a random-normal m x n input and a
random-normal k x k kernel per layer shape; the workloads here keep that
recipe (or a uniform input where stated) at larger shapes and with a batch of
vectors that share one T.  Batches are stored batch-minor: element
(pixel q, column c) sits at q*batch + c.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    m: int
    n: int
    k: int
    s: int
    p: int
    batch: int
    x_dist: str          # "uniform" = U(-1, 1), "normal" = N(0, 1)
    k_std: float         # kernel ~ N(0, k_std**2)
    seed: int

    @property
    def shape(self):
        return (self.m, self.n, self.k, self.s, self.p)


WORKLOADS = {w.name: w for w in [
    Workload("small_32_k3",        32,   32,   3, 1, 1, 1,   "uniform", 1.0,       0),
    Workload("strided_256_k5_b64", 256,  256,  5, 2, 2, 64,  "uniform", 1.0,       2),
    Workload("headline_1024_k7_b1", 1024, 1024, 7, 1, 3, 1,  "normal",  1.0 / 7.0, 3),
    Workload("headline_1024_k7_b16", 1024, 1024, 7, 1, 3, 16, "normal", 1.0 / 7.0, 3),
    Workload("cnn_224_k3_b256",    224,  224,  3, 1, 1, 256, "normal",  1.0 / 3.0, 4),
    Workload("padheavy_512_k9_s3", 512,  512,  9, 3, 8, 1,   "uniform", 1.0,       5),
    Workload("padheavy_4096_k11_s4_b4", 4096, 4096, 11, 4, 5, 4, "uniform", 1.0,   6),
]}

HEADLINE = "headline_1024_k7_b16"


def make_kernel(k: int, k_std: float, seed: int) -> np.ndarray:
    """k*k float32 kernel, row-major, N(0, k_std^2)."""
    rng = np.random.default_rng([seed, 0x4B])
    return (rng.standard_normal(k * k) * k_std).astype(np.float32)


def make_input(m: int, n: int, batch: int, dist: str, seed: int) -> np.ndarray:
    """m*n*batch float32 values, batch-minor."""
    rng = np.random.default_rng([seed, 0x58])
    size = m * n * batch
    if dist == "uniform":
        return rng.uniform(-1.0, 1.0, size).astype(np.float32)
    if dist == "normal":
        return rng.standard_normal(size, dtype=np.float32)
    raise ValueError("unknown distribution %r" % dist)


def make(w: Workload):
    """(x, K) host arrays for a workload."""
    return make_input(w.m, w.n, w.batch, w.x_dist, w.seed), make_kernel(w.k, w.k_std, w.seed)


def densenet121_layer_shapes():
    """The 123 single-channel layer shapes (m, n, k, s, p) of the paper's
    Table 2, in the table's reading order (down each column, then across).
    The table as printed has no block2.layer1.conv1 row; it is kept as printed."""
    conv1 = lambda e: (e, e, 1, 1, 0)
    conv3 = lambda e: (e, e, 3, 1, 1)
    pool2 = lambda e: (e, e, 2, 2, 0)
    shapes = [(224, 224, 7, 2, 3), (112, 112, 3, 2, 1)]
    shapes += [conv1(56), conv3(56)] * 6 + [conv1(56), pool2(56)]
    shapes += [conv3(28)] + [conv1(28), conv3(28)] * 11 + [conv1(28), pool2(28)]
    shapes += [conv1(14), conv3(14)] * 24 + [conv1(14), pool2(14)]
    shapes += [conv1(7), conv3(7)] * 16
    return shapes


def densenet121_sweep(batch: int = 1, seed: int = 121):
    """The paper's experiment (Section 4.1): for every layer shape of Table 2 a
    random-normal input and a random-normal kernel.  Yields (shape, x, K) per
    layer, each layer with its own draws."""
    for idx, (m, n, k, s, p) in enumerate(densenet121_layer_shapes()):
        rng = np.random.default_rng([seed, idx])
        x = rng.standard_normal(m * n * batch, dtype=np.float32)
        K = rng.standard_normal(k * k, dtype=np.float32)
        yield (m, n, k, s, p), x, K


def march_edge_grid(transposed: bool = False, every: int = 3):
    """Small shapes at the edge of what the strip-marching apply kernels accept, as
    ((m, n, k, s, p), batch) pairs: one to a few result lines, strips with ragged ends, every
    padding from none to beyond the kernel (empty rows, k > m, slide remainders).  Result lines
    must hold at least 32 pixels and rows at least 16 entries (k >= 4 for T; ceil(k/s) >= 4 for
    the transposed matrix, whose result lines are the input lines).  Every `every`-th shape of
    the full product is kept (the stride is coprime to the loop lengths), batches 1, 4, 8, 16
    in turn."""
    ms = (1, 2, 3, 9, 17, 33)
    ns = tuple(range(30, 41)) + tuple(range(63, 67)) + tuple(range(127, 131))
    ks = (4, 5, 7, 9, 11)
    batches = (1, 4, 8, 16)
    idx = kept = 0
    for m in ms:
        for n in ns:
            for k in ks:
                for s in (1, 2, 3):
                    for p in range(0, k + 2):
                        if k > m + 2 * p or k > n + 2 * p:
                            continue
                        if transposed:
                            if n < 32 or -(-k // s) < 4:
                                continue
                        elif (n + 2 * p - k) // s + 1 < 32:
                            continue
                        idx += 1
                        if idx % every:
                            continue
                        yield (m, n, k, s, p), batches[kept % 4]
                        kept += 1
