"""A plain elementwise pass of known size (dst = src + 1: SIZE bytes read, SIZE written).

Run under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE) to learn what those counters read
for a kernel whose HBM traffic is known exactly (SIZE bytes read, SIZE bytes written); the
ratio is the scale factor applied to the same counters measured on the scan kernel.
"""
import sys

import torch

SIZE = 1 << 30  # bytes copied per launch (larger than the 256 MB last-level cache)


def main():
    reps = int(sys.argv[1]) if len(sys.argv) > 1 else 3
    src = torch.empty(SIZE // 4, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(reps):
        torch.add(src, 1.0, out=dst)
    torch.cuda.synchronize()
    print(f"copied {SIZE} bytes x {reps}")


if __name__ == "__main__":
    main()
