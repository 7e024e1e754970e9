"""What would residual-PQ landmarks buy?  A float64 emulation of the scan rule, on the CPU.

The paper's PQ integration (Section 4.2) takes its landmarks from a product quantiser; it does not
say whether the quantiser codes the vectors or their residuals to the coarse centroid of their
list.  This script indexes a scaled-down workload both ways (same lists, same training sample,
codebooks trained on the raw vectors / on the residuals) and runs Section 4.2's rule (seed of k,
batches of B, survive <=> Equation 3's bound <= the k-th distance) in float64 with each kind of
landmark, for a range of gamma.  It prints, per gamma: recall@k against the exact neighbours,
exact distances per query, and the share of candidates whose partial landmark distance over the
first 8 subspaces alone already exceeds (Gamma(l,x) + sqrt(tau))^2 at the final threshold (what
an early-abandoning scan can stop after 8 code bytes).

A study, not a test (pytest does not collect it): it calls the oracle's index routines and the
seeded input generators only, never the HIP path.

    python tests/residual_landmark_study.py [workload=C2] [n=100000] [queries=100]
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from oracle import index_build, trim_oracle          # noqa: E402
from paper_2508_17828_amd import synth               # noqa: E402


def sq_dists(q64, x):
    """[nq][n] squared distances in float64 (expanded form; a study, not a decision)."""
    x64 = x.astype(np.float64)
    d = (q64 * q64).sum(1)[:, None] - 2.0 * (q64 @ x64.T) + (x64 * x64).sum(1)[None, :]
    return np.maximum(d, 0.0)


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "C2"
    n = int(sys.argv[2]) if len(sys.argv) > 2 else 100_000
    nq = int(sys.argv[3]) if len(sys.argv) > 3 else 100
    w0 = synth.WORKLOADS[name]
    scale = n / w0.n
    nlist = max(8, int(round(w0.nlist * scale)))
    w = synth.scaled(w0, n, nq, ncomp=max(8, int(round(w0.ncomp * scale))), nlist=nlist,
                     nprobe=min(w0.nprobe, nlist))
    base = synth.base_vectors(w)
    queries = synth.query_vectors(w)
    tr, init = synth.kmeans_draws(w, 64 * w.nlist, w.nlist, stream=1)
    cent, _ = index_build.kmeans(base[tr], w.nlist, w.kmeans_iters, init)
    ids, offs = index_build.ivf_assign(base, cent)
    base = np.ascontiguousarray(base[ids])
    lst = np.repeat(np.arange(w.nlist), np.diff(offs))
    probes = trim_oracle.ivf_probe(queries, cent, w.nprobe)
    _, init = synth.kmeans_draws(w, 16384, 256, stream=0)
    trows = np.random.default_rng(5).choice(n, min(n, 16384), replace=False)

    def landmarks(vectors):
        cb = index_build.train_pq(vectors[trows], w.M, w.kmeans_iters, init)
        codes, dlx = trim_oracle.encode(vectors, cb)
        dec = np.concatenate([cb[j][codes[:, j]] for j in range(w.M)], axis=1)
        return dec.astype(np.float32), dlx.astype(np.float64)

    L_raw, b_raw = landmarks(base)
    D_res, b_res = landmarks((base - cent[lst]).astype(np.float32))
    L_res = D_res + cent[lst]
    print(f"{name} scaled to n={n}: {w.nlist} lists, {w.nprobe} probed, PQ {w.M}x256, k={w0.k}, B={w0.batch}; "
          f"mean landmark distance: raw codes {b_raw.mean():.4g}, residual codes {b_res.mean():.4g}", flush=True)
    k, B = w0.k, w0.batch
    d8 = 8 * (w.d // w.M)
    q64 = queries.astype(np.float64)
    d2_all = sq_dists(q64, base)
    truth = np.argsort(d2_all, axis=1, kind="stable")[:, :k]
    cand = [np.concatenate([np.arange(offs[l], offs[l + 1]) for l in probes[i]]) for i in range(nq)]
    per_kind = {}
    for kind, L, b in (("raw", L_raw, b_raw), ("residual", L_res, b_res)):
        per_kind[kind] = (np.sqrt(sq_dists(q64, L)), sq_dists(q64[:, :d8], L[:, :d8]), b)
    for gamma in (0.0, 0.2, 0.3, 0.4, 0.45, 0.5, 0.6, 0.7, 0.8):
        row = [f"gamma {gamma:4.2f}:"]
        for kind in ("raw", "residual"):
            a_all, p8_all, b = per_kind[kind]
            nex = hits = stop8 = tot = 0
            for i in range(nq):
                pos = cand[i]
                d2, a, bb = d2_all[i, pos], a_all[i, pos], b[pos]
                g = (a - bb) ** 2 + 2.0 * gamma * a * bb
                keep = sorted(zip(d2[:k], pos[:k]))
                cnt, at = min(k, len(pos)), k
                while at < len(pos):
                    tau = keep[k - 1][0] if len(keep) >= k else np.inf
                    end = min(at + B, len(pos))
                    m = g[at:end] <= tau
                    cnt += int(m.sum())
                    keep = sorted(keep + list(zip(d2[at:end][m], pos[at:end][m])))[:k]
                    at = end
                tau = keep[-1][0]
                stop8 += int((p8_all[i, pos] > (bb + np.sqrt(tau)) ** 2).sum())
                tot += len(pos)
                hits += len(set(truth[i].tolist()) & {p for _, p in keep})
                nex += cnt
            row.append(f"{kind}: recall {hits / (nq * k):.3f}, exact/query {nex / nq:.0f}, stop after 8 bytes {stop8 / tot:.3f};")
        print(" ".join(row), flush=True)


if __name__ == "__main__":
    main()
