"""Times index construction with libtrim's kernels on a workload: PQ codebook training,
coarse-centroid training, coarse assignment of the base set, encoding and the scan layouts;
run it under rocprofv3 for the per-kernel split."""
import sys
import time

import numpy as np
import torch

from paper_2508_17828_amd import synth, trim


def timed(label, fn):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    out = fn()
    torch.cuda.synchronize()
    print(f"{label:34s} {1e3 * (time.perf_counter() - t0):10.2f} ms", flush=True)
    return out


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "C2"
    w = synth.WORKLOADS[name]
    base = torch.from_numpy(synth.base_vectors(w)).cuda()
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    tr, init = synth.kmeans_draws(w, 65536, 256, stream=0)
    train = base[dev(tr)].contiguous()
    init_t = dev(init.astype(np.int32))
    trim.trim_train_pq(train, w.M, 1, init_t)          # warm-up (code load)
    cb = timed(f"train_pq {train.shape[0]} rows x{w.kmeans_iters} iters", lambda: trim.trim_train_pq(train, w.M, w.kmeans_iters, init_t))
    if w.nlist:
        tr, init = synth.kmeans_draws(w, 64 * w.nlist, w.nlist, stream=1)
        xt = base[dev(tr)].contiguous()
        init_l = dev(init.astype(np.int32))
        cen = timed(f"train_ivf {xt.shape[0]} rows x{w.kmeans_iters} iters", lambda: trim.trim_train_ivf(xt, w.nlist, w.kmeans_iters, init_l))
        timed(f"coarse assignment of {w.n} rows", lambda: trim.trim_ivf_probe(base, cen, 1))
    codes, dlx = timed(f"encode {w.n} rows", lambda: trim.trim_encode(base, cb))
    if w.M % 8 == 0:
        timed("scan head", lambda: trim.trim_pack_scan_head(codes, dlx))
    if w.M % 16 == 0:
        timed("tiled codes", lambda: trim.trim_pack_codes_tiled(codes))


if __name__ == "__main__":
    main()
