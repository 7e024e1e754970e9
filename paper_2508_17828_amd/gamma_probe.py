"""Runs the confidence-level route of Section 3.2 on a workload: gamma(p) from sampled data
vectors and queries (trim_estimate_gamma), its cost, and the recall / pruning ratio that a kNN
search with that gamma reaches."""
import sys

import numpy as np
import torch

from paper_2508_17828_amd import index_setup, synth, trim


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "C2"
    S = int(sys.argv[2]) if len(sys.argv) > 2 else 1000
    w = synth.WORKLOADS[name]
    bw = index_setup.build_workload(w)
    ix, queries = bw.index, bw.queries
    rows = torch.from_numpy(np.sort(synth.sample_indices(6000 + w.seed, 0, w.n, S)).astype(np.int32)).cuda()
    # the sample queries are fresh draws from the query law, not the evaluation queries
    ws = synth.scaled(w, w.n, min(w.nq, 10_000), seed=w.seed + 100)
    sq = torch.from_numpy(synth.query_vectors(ws)).cuda()
    pr = trim.trim_ivf_probe(queries, bw.centroids, w.nprobe) if w.nlist else None
    nt = min(1000, w.nq)
    truth = trim.trim_search_knn(ix, queries[:nt].contiguous(), w.k, 0.0, 4096, want_stats=False)["ids"]
    for p in (1.0, 0.999, 0.99, 0.95, 0.9):
        trim.trim_estimate_gamma(ix, rows, sq, p)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g, gx = trim.trim_estimate_gamma(ix, rows, sq, p)
        e1.record()
        torch.cuda.synchronize()
        gamma = float(g.item())
        r = trim.trim_search_knn(ix, queries, w.k, gamma, w.batch, probes=pr)
        rec = index_setup.recall_at_k(r["ids"][:nt], truth)
        prune = 1.0 - r["n_exact"].sum().item() / max(1, r["n_scanned"].sum().item())
        print(f"p={p:<6} gamma={gamma:.4f} (median gamma_x {gx.median().item():.4f})  "
              f"estimate {e0.elapsed_time(e1):.2f} ms for {S} x {sq.shape[0]} pairs   "
              f"recall@{w.k}={rec:.4f} pruning={prune:.5f}", flush=True)


if __name__ == "__main__":
    main()
