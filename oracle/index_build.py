"""Index construction for the oracle side (test infrastructure): k-means codebooks and
IVF lists.  The paper only says PQ/IVF are trained by k-means with t iterations
(Section 3.1, cost O(mCn(d/m)t); Section 6.1, C = 256, C' coarse lists); any valid
codebook is acceptable data for both the oracle scan and the GPU scan, so the numeric
values produced here are "parity unpinned"; what is pinned is Lloyd's invariant (the
objective never increases) and determinism.

Random choices (training rows, initial centroids) are inputs, never drawn here.
Distances inside k-means use a library matmul in float64 (a library primitive as a step).

train_pq_fixed / train_ivf_fixed are the same Lloyd iterations with every rounding fixed, so
that a second implementation can reproduce the centroids bit for bit: the assignment step
is the binary32 nearest-centroid rule of the index itself (trim_oracle.encode for a PQ
subspace, trim_oracle.ivf_probe with one probe for the coarse lists: smallest index on
ties), and a centroid is the float64 sum of its member rows, added in ascending row order,
divided by their number and rounded once to binary32; an empty cluster keeps its centroid.
"""
from __future__ import annotations

import numpy as np


def _assign(x64: np.ndarray, c64: np.ndarray):
    """Nearest centroid per row (smallest index on ties) and its squared distance."""
    out_a = np.empty(x64.shape[0], dtype=np.int64)
    out_d = np.empty(x64.shape[0], dtype=np.float64)
    cn = (c64 * c64).sum(axis=1)
    step = max(1, (1 << 24) // max(1, c64.shape[0]))
    for lo in range(0, x64.shape[0], step):
        xs = x64[lo:lo + step]
        dist = (xs * xs).sum(axis=1)[:, None] - 2.0 * (xs @ c64.T) + cn[None, :]
        a = np.argmin(dist, axis=1)
        out_a[lo:lo + step] = a
        out_d[lo:lo + step] = dist[np.arange(xs.shape[0]), a]
    return out_a, out_d


def kmeans(train: np.ndarray, K: int, iters: int, init_rows: np.ndarray):
    """Lloyd's algorithm.  Returns (centroids float32 [K][dim], objective per iteration).

    Initial centroids are train[init_rows]; an empty cluster keeps its previous
    centroid; a centroid is the float64 mean of its members rounded to float32.
    objective[i] is the mean squared distance to the nearest centroid measured at the
    start of iteration i (before that iteration's update).
    """
    assert init_rows.shape[0] == K
    x64 = train.astype(np.float64)
    cent = train[init_rows].astype(np.float32)
    objective = []
    for _ in range(iters):
        a, dmin = _assign(x64, cent.astype(np.float64))
        objective.append(float(dmin.mean()))
        sums = np.zeros((K, x64.shape[1]), dtype=np.float64)
        np.add.at(sums, a, x64) if x64.shape[0] < 4096 else _scatter_sum(sums, a, x64)
        cnt = np.bincount(a, minlength=K)
        nz = cnt > 0
        cent[nz] = (sums[nz] / cnt[nz, None]).astype(np.float32)
    return cent, objective


def _scatter_sum(sums, a, x64):
    order = np.argsort(a, kind="stable")
    a_s = a[order]
    starts = np.flatnonzero(np.r_[True, a_s[1:] != a_s[:-1]])
    sums[a_s[starts]] = np.add.reduceat(x64[order], starts, axis=0)


def train_pq(train: np.ndarray, M: int, iters: int, init_rows: np.ndarray, ncent: int = 256) -> np.ndarray:
    """PQ codebooks [M][ncent][d/M]: one k-means per subspace (Section 2.2); ncent = 256 for
    8-bit codes, 16 for the 4-bit codes of the FastScan variant (Section 6.1)."""
    d = train.shape[1]
    dsub = d // M
    cb = np.empty((M, ncent, dsub), dtype=np.float32)
    for j in range(M):
        cb[j], _ = kmeans(np.ascontiguousarray(train[:, j * dsub:(j + 1) * dsub]), ncent,
                          iters, init_rows[:ncent])
    return cb


def ivf_assign(base: np.ndarray, centroids: np.ndarray):
    """Coarse assignment of every base vector, then list-contiguous storage order.

    Returns (order, list_offsets): order[p] = original id stored at position p (ascending
    id inside a list), list_offsets int64 [nlist+1].
    """
    nlist = centroids.shape[0]
    c64 = centroids.astype(np.float64)
    a = np.empty(base.shape[0], dtype=np.int64)
    step = 1 << 15
    for lo in range(0, base.shape[0], step):
        a[lo:lo + step], _ = _assign(base[lo:lo + step].astype(np.float64), c64)
    order = np.argsort(a, kind="stable").astype(np.int32)
    counts = np.bincount(a, minlength=nlist)
    list_offsets = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(counts, out=list_offsets[1:])
    return order, list_offsets


def _update_fixed(x: np.ndarray, a: np.ndarray, cent: np.ndarray) -> np.ndarray:
    """Means in float64, rows added one by one in ascending row order."""
    K, dim = cent.shape
    sums = np.zeros((K, dim), dtype=np.float64)
    np.add.at(sums, a, x.astype(np.float64))       # unbuffered: sequential in row order
    cnt = np.bincount(a, minlength=K)
    out = cent.copy()
    nz = cnt > 0
    out[nz] = (sums[nz] / cnt[nz, None].astype(np.float64)).astype(np.float32)
    return out


def train_pq_fixed(train: np.ndarray, M: int, iters: int, init_rows: np.ndarray) -> np.ndarray:
    """PQ codebooks [M][256][d/M] by Lloyd iterations with the fixed roundings described in
    the header (Section 2.2: one k-means with 256 centroids per subspace)."""
    from . import trim_oracle
    ns, d = train.shape
    dsub = d // M
    assert init_rows.shape[0] == 256
    cb = np.ascontiguousarray(train[init_rows].reshape(256, M, dsub).transpose(1, 0, 2)).astype(np.float32)
    for _ in range(iters):
        codes, _ = trim_oracle.encode(train, cb)
        for j in range(M):
            cb[j] = _update_fixed(train[:, j * dsub:(j + 1) * dsub], codes[:, j].astype(np.int64), cb[j])
    return cb


def train_pq_fs_fixed(train: np.ndarray, m: int, iters: int, init_rows: np.ndarray) -> np.ndarray:
    """Codebooks [m][16][d/m] for 4-bit codes (Section 6.1: FastScan variants, m = d/2) by the
    same Lloyd iterations with fixed roundings; the assignment is trim_oracle_fs.encode's."""
    from . import trim_oracle_fs
    ns, d = train.shape
    dsub = d // m
    assert init_rows.shape[0] == 16
    cb = np.ascontiguousarray(train[init_rows].reshape(16, m, dsub).transpose(1, 0, 2)).astype(np.float32)
    for _ in range(iters):
        codes, _ = trim_oracle_fs.encode(train, cb)
        nib = trim_oracle_fs.unpack(codes, m)
        for j in range(m):
            cb[j] = _update_fixed(train[:, j * dsub:(j + 1) * dsub], nib[:, j].astype(np.int64), cb[j])
    return cb


def train_ivf_fixed(train: np.ndarray, nlist: int, iters: int, init_rows: np.ndarray) -> np.ndarray:
    """Coarse centroids [nlist][d] (Section 6.1: C' lists), same fixed roundings."""
    from . import trim_oracle
    assert init_rows.shape[0] == nlist
    cent = np.ascontiguousarray(train[init_rows]).astype(np.float32)
    for _ in range(iters):
        a = trim_oracle.ivf_probe(train, cent, 1)[:, 0].astype(np.int64)
        cent = _update_fixed(train, a, cent)
    return cent
