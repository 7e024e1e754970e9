"""Machine ceilings the scan is priced against, measured with the library's own aids:
the streaming-read rate of HBM (a 4 GiB buffer read once per launch) and the rate of table
lookups out of on-chip memory (the scan's lookup-and-add sequence with nothing else going on),
each at several grid sizes; the best of each is the ceiling.  Prints one JSON line.
"""
import json
import sys

import torch

from paper_2508_17828_amd import trim


def _time(fn, reps):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e-3 / reps


def main():
    reps = int(sys.argv[1]) if len(sys.argv) > 1 else 10
    size = 4 << 30
    buf = torch.empty(size // 4, dtype=torch.int32, device="cuda").random_()
    sink = torch.empty(8192, dtype=torch.int32, device="cuda")
    read = {}
    for blocks in (512, 768, 1024, 2048, 4096, 8192):
        t = _time(lambda: trim.trim_ceiling_stream_read(buf, blocks, sink), reps)
        read[blocks] = round(size / t / 1e9, 1)
    del buf
    iters = 2048
    fsink = torch.empty(2048 * 512, dtype=torch.float32, device="cuda")
    look = {}
    for blocks in (256, 512, 768, 1024, 2048):      # 1..4 workgroups per CU, then two rounds
        t = _time(lambda: trim.trim_ceiling_lds_gather(blocks, iters, 12345, fsink), reps)
        look[blocks] = round(blocks * 512 * iters * 32 / t / 1e9, 1)
    wide = {}
    for ef in (2, 4):                                   # entries of 2 and 4 values, 1024 workgroups
        t = _time(lambda: trim.trim_ceiling_lds_gather(1024, iters, 12345, fsink, entry_floats=ef), reps)
        wide[ef] = round(1024 * 512 * iters * 8 / t / 1e9, 1)
    print(json.dumps({
        "stream_read_GBps_by_blocks": read, "stream_read_GBps": max(read.values()),
        "lds_Glookups_per_s_by_blocks": look, "lds_Glookups_per_s": max(look.values()),
        "lds_wave_instructions_per_s": round(max(look.values()) * 1e9 / 64, -8),
        "lds_Glookups_per_s_entries_of_2_and_4_values": wide,
    }))


if __name__ == "__main__":
    main()
