"""Shared by the tests: build an index for a synthetic workload with the ORACLE
(k-means codebooks, codes, landmark distances, IVF lists, probes), as plain arrays that
both the oracle scan and the GPU scan consume as data."""
from __future__ import annotations

import functools

import numpy as np

from oracle import index_build, trim_oracle, trim_oracle_fs
from paper_2508_17828_amd import synth


class Built:
    def __init__(self, w, index, queries, probes, centroids):
        self.w, self.index, self.queries, self.probes, self.centroids = \
            w, index, queries, probes, centroids


def build(w: synth.Workload, pq_train_max=16384, ivf_train_per_list=64, encode=True) -> Built:
    base = synth.base_vectors(w)
    queries = synth.query_vectors(w)
    tr, init = synth.kmeans_draws(w, pq_train_max, 256, stream=0)
    codebooks = index_build.train_pq(base[tr], w.M, w.kmeans_iters, init)
    ids = list_offsets = centroids = probes = None
    if w.nlist:
        tr, init = synth.kmeans_draws(w, ivf_train_per_list * w.nlist, w.nlist, stream=1)
        centroids, _ = index_build.kmeans(base[tr], w.nlist, w.kmeans_iters, init)
        ids, list_offsets = index_build.ivf_assign(base, centroids)
        base = np.ascontiguousarray(base[ids])
        probes = trim_oracle.ivf_probe(queries, centroids, w.nprobe)
    if encode:
        codes, dlx = trim_oracle.encode(base, codebooks)
    else:
        codes = np.zeros((w.n, w.M), np.uint8)
        dlx = np.zeros(w.n, np.float32)
    ix = trim_oracle.Index(base, codes, dlx, codebooks, ids=ids, list_offsets=list_offsets,
                           centroids=centroids)
    return Built(w, ix, queries, probes, centroids)


@functools.lru_cache(maxsize=8)
def cached(name: str, n: int = 0, nq: int = 0, nlist: int = -1, nprobe: int = -1) -> Built:
    w = synth.WORKLOADS[name]
    kw = {}
    if nlist >= 0:
        kw["nlist"] = nlist
    if nprobe >= 0:
        kw["nprobe"] = nprobe
    if n or nq or kw:
        w = synth.scaled(w, n or w.n, nq or w.nq, **kw)
    return build(w)


def radius_at_percentile(b: Built, percent: float, nq_s=64, nb_s=2048) -> float:
    """Unsquared radius with `percent` % of sampled query-base pairs inside (float64)."""
    qi, bi = synth.pair_sample(b.w, nq_s, nb_s)
    q = b.queries[qi].astype(np.float64)
    x = b.index.base[bi].astype(np.float64)
    d2 = ((q * q).sum(1)[:, None] - 2 * q @ x.T + (x * x).sum(1)[None, :]).ravel()
    return float(np.sqrt(max(np.percentile(d2, percent), 0.0)))


def build_fs(w: synth.Workload, pq_train_max=16384, ivf_train_per_list=64) -> Built:
    """The same workload indexed with 4-bit codes: m = d/2 subspaces of 16 centroids
    (Section 6.1, FastScan variants); everything else as build()."""
    base = synth.base_vectors(w)
    queries = synth.query_vectors(w)
    m = w.d // 2
    tr, init = synth.kmeans_draws(w, pq_train_max, 256, stream=0)
    codebooks = index_build.train_pq(base[tr], m, w.kmeans_iters, init, ncent=16)
    ids = list_offsets = centroids = probes = None
    if w.nlist:
        tr, init = synth.kmeans_draws(w, ivf_train_per_list * w.nlist, w.nlist, stream=1)
        centroids, _ = index_build.kmeans(base[tr], w.nlist, w.kmeans_iters, init)
        ids, list_offsets = index_build.ivf_assign(base, centroids)
        base = np.ascontiguousarray(base[ids])
        probes = trim_oracle.ivf_probe(queries, centroids, w.nprobe)
    codes, dlx = trim_oracle_fs.encode(base, codebooks)
    ix = trim_oracle_fs.Index(base, codes, dlx, codebooks, ids=ids, list_offsets=list_offsets,
                              centroids=centroids)
    return Built(w, ix, queries, probes, centroids)


@functools.lru_cache(maxsize=8)
def cached_fs(name: str, n: int = 0, nq: int = 0, nlist: int = -1, nprobe: int = -1) -> Built:
    w = synth.WORKLOADS[name]
    kw = {}
    if nlist >= 0:
        kw["nlist"] = nlist
    if nprobe >= 0:
        kw["nprobe"] = nprobe
    if n or nq or kw:
        w = synth.scaled(w, n or w.n, nq or w.nq, **kw)
    return build_fs(w)
