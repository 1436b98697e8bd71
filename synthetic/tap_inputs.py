"""Seeded, synthetic sample pools for the calibration-set clustering.

Nothing here computes any step of the clustering: the functions only describe
workload shapes and draw random tensors and index sets.  They stand in for the
pool of intermediate samples that the paper collects from a pre-trained DiT
over the ImageNet classes during sampling (Experimental Settings section): the
shapes are real (a 256^2 latent flattened to 4 x 32 x 32 = 4096 features, a
timestamp per sample, 1/20 of the pool per subsample, three subsamples, 100
clusters), the values are random draws with the structure such a pool has (a
class-dependent signal that fades into noise as the timestep grows).
"""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np


@dataclass(frozen=True)
class TapWorkload:
    name: str
    N: int              # pool size
    F: int              # features per sample
    n: int              # samples per subsample
    m: int              # subsamples
    k: int              # clusters
    alpha: float        # weight of the spatial similarity
    steps: int          # sampler steps the pool is drawn from
    classes: int
    seed: int


TAP_WORKLOADS = {
    # the small case the oracle finishes in seconds
    "tap0": TapWorkload("tap0", N=1536, F=256, n=160, m=3, k=8, alpha=0.5, steps=50, classes=16, seed=500),
    # the paper's setting: three subsamples of 1/20 of the pool, 100 clusters, 256^2 latents, 50 steps
    "tap1": TapWorkload("tap1", N=32768, F=4096, n=1638, m=3, k=100, alpha=0.5, steps=50, classes=1000, seed=510),
}


def make_pool(N: int, F: int, steps: int, classes: int, seed: int):
    """(X [N, F] float32, t [N] float32 in [0, 1), class [N], step [N]): sample r is the signal of its class scaled
    by sqrt(abar(step)) plus Gaussian noise scaled by sqrt(1 - abar(step)), abar falling from 1 to 0 over the steps
    (the marginal a diffusion sampler's intermediate samples have)."""
    rng = np.random.default_rng(seed)
    proto = rng.standard_normal((classes, F)).astype(np.float32)
    cls = rng.integers(0, classes, size=N)
    step = rng.integers(0, steps, size=N)
    abar = np.cos(0.5 * np.pi * (step + 0.5) / steps) ** 2
    X = np.empty((N, F), dtype=np.float32)
    chunk = 4096
    for r0 in range(0, N, chunk):
        r1 = min(N, r0 + chunk)
        noise = rng.standard_normal((r1 - r0, F)).astype(np.float32)
        a = abar[r0:r1, None].astype(np.float32)
        X[r0:r1] = np.sqrt(a) * proto[cls[r0:r1]] + np.sqrt(1 - a) * noise
    t = (step / steps).astype(np.float32)
    return X, t, cls, step


def make_planted(N: int, F: int, k: int, seed: int, noise: float = 0.05, time_jitter: float = 0.01):
    """(X, t, truth [N]): k well separated groups; group g has its own random direction and its own time, samples
    scatter a little around both.  Group sizes are ragged (between half and one and a half of N / k)."""
    rng = np.random.default_rng(seed)
    w = rng.uniform(0.5, 1.5, size=k)
    sizes = np.maximum(1, np.floor(w / w.sum() * N).astype(int))
    sizes[0] += N - sizes.sum()
    truth = np.repeat(np.arange(k), sizes)
    rng.shuffle(truth)
    dirs = rng.standard_normal((k, F)).astype(np.float32)
    X = dirs[truth] + noise * rng.standard_normal((N, F)).astype(np.float32)
    t = ((truth + 0.5) / k + time_jitter * rng.standard_normal(N)).astype(np.float32)
    return X.astype(np.float32), t, truth


def make_subsamples(N: int, n: int, m: int, seed: int):
    """[m, n] int32: m draws of n distinct pool indices, each sorted ascending."""
    rng = np.random.default_rng(seed)
    return np.stack([np.sort(rng.choice(N, size=n, replace=False)) for _ in range(m)]).astype(np.int32)


def make_init(N: int, k: int, m: int, seed: int):
    """[m, k] int32: pool indices whose embedding rows start the k-means centres (distinct within a row)."""
    rng = np.random.default_rng(seed)
    return np.stack([rng.choice(N, size=k, replace=False) for _ in range(m)]).astype(np.int32)


def make_start_block(kb: int, n: int, seed: int):
    """[kb, n] float32 Gaussian start vectors for an iterative eigen-solver."""
    return np.random.default_rng(seed).standard_normal((kb, n)).astype(np.float32)
