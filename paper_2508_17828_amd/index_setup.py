"""Workload set-up on the GPU: train PQ / IVF centroids and lay the base set out in
list order, then encode it with libtrim.

Centroid training (Lloyd's k-means; the paper: Section 3.1, cost O(mCn(d/m)t), and
Section 6.1, C = 256 centroids per subspace, C' coarse lists) is preparation of the
index that the scan consumes, not part of the timed scan.  It is written with torch
tensor ops purely as a convenience for building benchmark inputs; codes, landmark
distances, probe selection and everything timed go through libtrim's kernels.
"""
from __future__ import annotations

import numpy as np
import torch

from . import synth, trim


def _lloyd(x: torch.Tensor, init: torch.Tensor, iters: int) -> torch.Tensor:
    """Batched Lloyd iterations.  x [G][ns][dim], init [G][K][dim] -> centroids [G][K][dim]."""
    cen = init.clone()
    G, ns, dim = x.shape
    K = cen.shape[1]
    xn = (x * x).sum(-1, keepdim=True)
    ar = torch.arange(G, device=x.device)[:, None].expand(G, ns)
    for _ in range(iters):
        dist = xn - 2.0 * torch.bmm(x, cen.transpose(1, 2)) + (cen * cen).sum(-1)[:, None, :]
        a = dist.argmin(-1)                                       # [G][ns]
        flat = (ar * K + a).reshape(-1)
        sums = torch.zeros((G * K, dim), device=x.device, dtype=torch.float64)
        sums.index_add_(0, flat, x.reshape(-1, dim).double())
        cnt = torch.bincount(flat, minlength=G * K).double()[:, None]
        new = (sums / cnt.clamp(min=1.0)).float().reshape(G, K, dim)
        cen = torch.where((cnt > 0).reshape(G, K, 1), new, cen)
    return cen


def _assign(x: torch.Tensor, cen: torch.Tensor, chunk: int = 1 << 16) -> torch.Tensor:
    out = torch.empty((x.shape[0],), dtype=torch.int64, device=x.device)
    cn = (cen * cen).sum(-1)[None, :]
    for lo in range(0, x.shape[0], chunk):
        xs = x[lo:lo + chunk]
        dist = (xs * xs).sum(-1, keepdim=True) - 2.0 * (xs @ cen.T) + cn
        out[lo:lo + chunk] = dist.argmin(-1)
    return out


class BuiltWorkload:
    def __init__(self, w, index, queries, centroids):
        self.w, self.index, self.queries, self.centroids = w, index, queries, centroids


def build_workload(w: synth.Workload, device: str = "cuda:0", pq_train: int = 65536,
                   ivf_train_per_list: int = 64) -> BuiltWorkload:
    """Generate the synthetic base set and queries, train centroids, store the base set in
    list order and encode it.  Returns device-resident tensors."""
    base_h = synth.base_vectors(w)
    queries = torch.from_numpy(synth.query_vectors(w)).to(device)
    base = torch.from_numpy(base_h).to(device)
    del base_h
    dsub = w.d // w.M
    tr, init = synth.kmeans_draws(w, pq_train, 256, stream=0)
    tr_t = torch.from_numpy(tr).to(device)
    xs = base[tr_t].reshape(tr.shape[0], w.M, dsub).permute(1, 0, 2).contiguous()
    init_t = torch.from_numpy(init).to(device)
    codebooks = _lloyd(xs, xs[:, init_t, :].contiguous(), w.kmeans_iters).contiguous()
    ids = list_offsets = centroids = None
    max_len = 0
    if w.nlist:
        tr, init = synth.kmeans_draws(w, ivf_train_per_list * w.nlist, w.nlist, stream=1)
        xt = base[torch.from_numpy(tr).to(device)]
        centroids = _lloyd(xt[None], xt[torch.from_numpy(init).to(device)][None],
                           w.kmeans_iters)[0].contiguous()
        a = _assign(base, centroids)
        order = torch.argsort(a, stable=True)
        counts = torch.bincount(a, minlength=w.nlist)
        list_offsets = torch.zeros((w.nlist + 1,), dtype=torch.int64, device=device)
        list_offsets[1:] = torch.cumsum(counts, 0)
        max_len = int(counts.max().item())
        base = base[order].contiguous()
        ids = order.to(torch.int32)
    codes, dlx = trim.trim_encode(base, codebooks)
    head = trim.trim_pack_scan_head(codes, dlx) if codes.shape[1] % 8 == 0 else None
    # long codes are also kept in the tiled layout (see trim_pack_codes_tiled)
    tiled = trim.trim_pack_codes_tiled(codes) if codes.shape[1] >= 64 and codes.shape[1] % 16 == 0 else None
    index = trim.Index(base, codes, dlx, codebooks, ids=ids, list_offsets=list_offsets,
                       max_list_len=max_len, scan_head=head, codes_tiled=tiled)
    return BuiltWorkload(w, index, queries, centroids)


def recall_at_k(found: torch.Tensor, truth: torch.Tensor) -> float:
    """Recall@k of Section 2.1: |R ∩ R'| / k averaged over queries (ids are unique per row)."""
    hit = (found[:, :, None] == truth[:, None, :]).any(-1)
    return float(hit.float().mean().item())
