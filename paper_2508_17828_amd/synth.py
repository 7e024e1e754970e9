"""Seeded synthetic inputs shaped like the paper's workloads (Table 1 shapes only).

This module only draws random vectors and random index choices. It holds none of
the method's arithmetic (no distances, no quantisation, no bounds), so both the
CPU oracle's callers and the HIP path's callers may use it to obtain identical
inputs. It imports neither of them.

The paper evaluates on public datasets (128-d SIFT-like, 960-d GIST-like,
1536-d text-embedding-like); none is available here, so Gaussian mixtures with
the same n / d stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

_CHUNK = 1 << 16


@dataclass(frozen=True)
class Workload:
    """One named configuration: data law, index parameters, search parameters."""

    name: str
    n: int
    nq: int
    d: int
    M: int
    ncomp: int
    law: str                      # "clip255" | "aniso01" | "unit"
    nlist: int = 0                # 0 => brute-force candidate scan
    nprobe: int = 0
    k: int = 10
    mode: str = "knn"             # "knn" | "range"
    gammas: Tuple[float, ...] = (0.0,)
    batch: int = 1024
    range_percentile: float = 0.0  # percent of sampled pair distances inside the radius
    seed: int = 0
    kmeans_iters: int = 10


WORKLOADS = {
    # 10k x 128, 64-component isotropic mixture, brute-force candidates.
    "C1": Workload("C1", 10_000, 100, 128, 16, 64, "clip255", k=10,
                   gammas=(0.0, 0.6), batch=256, seed=1),
    # 1M x 128 SIFT-like shape, IVF 1024 / nprobe 32, PQ 32x256.
    "C2": Workload("C2", 1_000_000, 10_000, 128, 32, 1024, "clip255", nlist=1024,
                   nprobe=32, k=10, gammas=(0.0, 0.5, 0.8), batch=1024, seed=2),
    # 1M x 960 GIST-like shape, brute-force scan with pruning, k=100.
    "C3": Workload("C3", 1_000_000, 1_000, 960, 120, 512, "aniso01", k=100,
                   gammas=(0.0, 0.7), batch=512, seed=3),
    # 1M x 1536 unit-norm embeddings, IVF 1024 / nprobe 64, range search.
    "C4": Workload("C4", 1_000_000, 10_000, 1536, 192, 256, "unit", nlist=1024,
                   nprobe=64, mode="range", gammas=(0.0, 0.7), range_percentile=0.1,
                   seed=4),
    # 10M x 128, IVF 4096 / nprobe 64, kNN k=10 plus a range pass.
    "C5": Workload("C5", 10_000_000, 10_000, 128, 32, 4096, "clip255", nlist=4096,
                   nprobe=64, k=10, gammas=(0.0, 0.5, 0.8), batch=1024,
                   range_percentile=0.01, seed=5),
    # Two more of the paper's dataset shapes (Table 1), as synthetic stand-ins like the rest:
    # 5M x 384 (the shape of its 384-dimensional image-descriptor set), IVF 4096 / nprobe 64
    # (Section 6.1: C' = 4096), PQ 48x256, kNN k=10;
    "T384": Workload("T384", 5_000_000, 10_000, 384, 48, 2048, "clip255", nlist=4096, nprobe=64,
                     k=10, gammas=(0.0, 0.5, 0.8), batch=1024, seed=6),
    # 2M x 768 unit-norm embeddings (the shape of its 768-dimensional text-embedding set),
    # IVF 2048 / nprobe 64, PQ 96x256, kNN k=10.
    "W768": Workload("W768", 2_000_000, 10_000, 768, 96, 512, "unit", nlist=2048, nprobe=64,
                     k=10, gammas=(0.0, 0.5, 0.8), batch=1024, seed=7),
}


def scaled(w: Workload, n: int, nq: int, **kw) -> Workload:
    """Same law and index shape as ``w`` with fewer vectors (for parity tests)."""
    from dataclasses import replace
    return replace(w, n=n, nq=nq, **kw)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream)])


def mixture_means(w: Workload) -> np.ndarray:
    """Component means of the workload's Gaussian mixture, float32 [ncomp][d]."""
    r = _rng(1000 + w.seed, 0)
    if w.law == "clip255":
        mu = r.uniform(0.0, 255.0, size=(w.ncomp, w.d))
    elif w.law == "aniso01":
        i = np.arange(1, w.d + 1, dtype=np.float64)
        u = r.uniform(0.0, 1.0, size=(w.ncomp, w.d))
        mu = 0.5 + 0.5 * (2.0 * u - 1.0) / np.sqrt(i)
    elif w.law == "unit":
        mu = r.standard_normal(size=(w.ncomp, w.d))
        mu /= np.linalg.norm(mu, axis=1, keepdims=True)
    else:
        raise ValueError(w.law)
    return mu.astype(np.float32)


def _draw(w: Workload, means: np.ndarray, count: int, stream: int,
          out: Optional[np.ndarray] = None) -> np.ndarray:
    r = _rng(1000 + w.seed, stream)
    if out is None:
        out = np.empty((count, w.d), dtype=np.float32)
    if w.law == "aniso01":
        sig = (0.1 / np.sqrt(np.arange(1, w.d + 1, dtype=np.float64))).astype(np.float32)
    for lo in range(0, count, _CHUNK):
        hi = min(count, lo + _CHUNK)
        comp = r.integers(0, w.ncomp, size=hi - lo)
        z = r.standard_normal(size=(hi - lo, w.d), dtype=np.float32)
        if w.law == "clip255":
            z *= np.float32(20.0)
            z += means[comp]
            np.clip(z, 0.0, 255.0, out=z)
        elif w.law == "aniso01":
            z *= sig
            z += means[comp]
            np.clip(z, 0.0, 1.0, out=z)
        else:  # unit
            z *= np.float32(1.0 / np.sqrt(w.d))
            z += means[comp]
            z /= np.linalg.norm(z, axis=1, keepdims=True)
        out[lo:hi] = z
    return out


def base_vectors(w: Workload, out: Optional[np.ndarray] = None) -> np.ndarray:
    """Base set, float32 [n][d], C-contiguous."""
    return _draw(w, mixture_means(w), w.n, 1, out)


def query_vectors(w: Workload) -> np.ndarray:
    """Queries, float32 [nq][d]: independent draws from the base set's mixture."""
    return _draw(w, mixture_means(w), w.nq, 2)


def sample_indices(seed: int, stream: int, n: int, count: int) -> np.ndarray:
    """``count`` distinct indices in [0, n), int64, in drawing order."""
    count = min(count, n)
    return _rng(seed, stream).choice(n, size=count, replace=False).astype(np.int64)


def kmeans_draws(w: Workload, n_train_max: int, K: int, stream: int):
    """Random choices a k-means run needs: (training-row indices, initial-centroid rows).

    Training rows are a seeded sample of at most ``n_train_max`` base rows; the
    initial centroids are K distinct rows of that sample (indices into it).
    """
    train = np.sort(sample_indices(3000 + w.seed, stream, w.n, n_train_max))
    init = sample_indices(3000 + w.seed, stream + 100_000, train.shape[0], K)
    return train, init


def pair_sample(w: Workload, nq_s: int, nb_s: int):
    """Seeded (query rows, base rows) used to place a range radius at a percentile."""
    qi = sample_indices(5000 + w.seed, 0, w.nq, nq_s)
    bi = sample_indices(5000 + w.seed, 1, w.n, nb_s)
    return qi, bi
