"""Times the stand-alone distance-table kernels (vector-ALU direct form and matrix-core
expanded form) on a workload's query set; run it under rocprofv3 for MFMA / HBM counters."""
import sys

import torch

from paper_2508_17828_amd import synth, trim


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "C2"
    reps = int(sys.argv[2]) if len(sys.argv) > 2 else 5
    w = synth.WORKLOADS[name]
    q = torch.from_numpy(synth.query_vectors(w)).cuda()
    g = torch.Generator(device="cuda").manual_seed(7)
    lo, hi = (0.0, 255.0) if w.law == "clip255" else (-1.0, 1.0)
    cb = torch.empty((w.M, 256, w.d // w.M), device="cuda").uniform_(lo, hi, generator=g)
    out = torch.empty((w.nq, w.M, 256), dtype=torch.float32, device="cuda")
    for mfma in (False, True):
        trim.trim_build_lut(q, cb, mfma=mfma, out=out)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            trim.trim_build_lut(q, cb, mfma=mfma, out=out)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        nbytes = out.numel() * 4
        flops = 3.0 * 256 * w.d * w.nq if not mfma else 2.0 * 256 * w.d * w.nq
        print(f"{name} table kernel mfma={int(mfma)}: {ms:.3f} ms, {nbytes / ms / 1e6:.0f} GB/s written "
              f"({nbytes / 1e6:.0f} MB), {flops / ms / 1e9:.2f} TFLOP/s")


if __name__ == "__main__":
    main()
