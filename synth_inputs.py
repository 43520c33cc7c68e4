"""Seeded synthetic inputs shared by the oracle-side and the HIP-side callers.

Holds none of the method's arithmetic: only the data a job would read from
its training set.  Images are N(0,1) in [N,H,W,C] float32, labels uniform
integers; gradient buffers for the stand-alone update benchmark are
N(0,1)*1e-2.  They stand in for the image-classification training sets the
paper's models were run on (its section 6 names TensorFlow's CNN benchmark
models, no dataset).
"""
import numpy as np


def dataset(seed: int, N: int, H: int, W: int, C: int, classes: int):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    y = rng.integers(0, classes, size=N, dtype=np.int32)
    return x, y


def gradient_buffers(seed: int, p: int, P: int):
    rng = np.random.default_rng(seed)
    return [(rng.standard_normal(P, dtype=np.float32) * np.float32(1e-2)) for _ in range(p)]


def vector(seed: int, n: int, scale: float = 1.0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(n, dtype=np.float32) * np.float32(scale)
