"""Workload set-up on the GPU: train PQ / IVF centroids, lay the base set out in list
order, encode it and pack the scan layouts, all with libtrim's kernels.

Centroid training (Lloyd's k-means; the paper: Section 3.1, cost O(mCn(d/m)t), and
Section 6.1, C = 256 centroids per subspace, C' coarse lists) is preparation of the
index that the scan consumes, not part of the timed scan.  torch is used here only to hold
the arrays and to sort / gather the base set into list order.
"""
from __future__ import annotations

import numpy as np
import torch

from . import synth, trim


class BuiltWorkload:
    def __init__(self, w, index, queries, centroids):
        self.w, self.index, self.queries, self.centroids = w, index, queries, centroids


def build_workload(w: synth.Workload, device: str = "cuda:0", pq_train: int = 65536,
                   ivf_train_per_list: int = 64, list_bounds: bool = True,
                   code_bits: int = 8) -> BuiltWorkload:
    """Generate the synthetic base set and queries, train centroids, store the base set in
    list order and encode it.  Returns device-resident tensors.  code_bits = 4: the index of
    the FastScan variant (Section 6.1: 4-bit codes, d/2 subspaces of 16 centroids) instead of
    the workload's M subspaces of 256."""
    base_h = synth.base_vectors(w)
    queries = torch.from_numpy(synth.query_vectors(w)).to(device)
    base = torch.from_numpy(base_h).to(device)
    del base_h
    tr, init = synth.kmeans_draws(w, pq_train, 256, stream=0)
    train = base[torch.from_numpy(tr).to(device)].contiguous()
    init_d = torch.from_numpy(init.astype(np.int32)).to(device)
    if code_bits == 4:
        codebooks = trim.trim_fs_train_pq(train, w.d // 2, w.kmeans_iters, init_d[:16].contiguous())
    else:
        codebooks = trim.trim_train_pq(train, w.M, w.kmeans_iters, init_d)
    del train
    ids = list_offsets = centroids = None
    max_len = 0
    if w.nlist:
        tr, init = synth.kmeans_draws(w, ivf_train_per_list * w.nlist, w.nlist, stream=1)
        xt = base[torch.from_numpy(tr).to(device)].contiguous()
        centroids = trim.trim_train_ivf(xt, w.nlist, w.kmeans_iters,
                                        torch.from_numpy(init.astype(np.int32)).to(device))
        a = trim.trim_ivf_probe(base, centroids, 1)[:, 0].long()
        order = torch.argsort(a, stable=True)
        counts = torch.bincount(a, minlength=w.nlist)
        list_offsets = torch.zeros((w.nlist + 1,), dtype=torch.int64, device=device)
        list_offsets[1:] = torch.cumsum(counts, 0)
        max_len = int(counts.max().item())
        base = base[order].contiguous()
        ids = order.to(torch.int32)
    codes, dlx = (trim.trim_fs_encode if code_bits == 4 else trim.trim_encode)(base, codebooks)
    head = trim.trim_pack_scan_head(codes, dlx) if codes.shape[1] % 8 == 0 else None
    # long codes are also kept in the tiled layout (see trim_pack_codes_tiled)
    tiled = trim.trim_pack_codes_tiled(codes) if codes.shape[1] >= 64 and codes.shape[1] % 16 == 0 else None
    index = trim.Index(base, codes, dlx, codebooks, ids=ids, list_offsets=list_offsets,
                       max_list_len=max_len, scan_head=head, codes_tiled=tiled, code_bits=code_bits)
    if list_offsets is not None and list_bounds:
        index.list_bounds = trim.trim_pack_list_bounds(index)
    return BuiltWorkload(w, index, queries, centroids)


def recall_at_k(found: torch.Tensor, truth: torch.Tensor) -> float:
    """Recall@k of Section 2.1: |R ∩ R'| / k averaged over queries (ids are unique per row)."""
    hit = (found[:, :, None] == truth[:, None, :]).any(-1)
    return float(hit.float().mean().item())
