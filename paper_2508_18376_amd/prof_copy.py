"""A plain device-to-device copy of known size, to calibrate rocprofv3's FETCH_SIZE / WRITE_SIZE
counters: run it under `rocprofv3 --pmc FETCH_SIZE` (then WRITE_SIZE) and compare what the counter
reads for the copy kernel with the bytes it is known to move.

    python3 paper_2508_18376_amd/prof_copy.py [MiB per buffer, default 1024] [repeats, default 3]
"""
import sys

import torch


def main() -> None:
    mib = int(sys.argv[1]) if len(sys.argv) > 1 else 1024
    reps = int(sys.argv[2]) if len(sys.argv) > 2 else 3
    n = mib * 1024 * 1024 // 4
    src = torch.arange(n, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(reps):
        dst.copy_(src)  # one elementwise copy kernel: reads mib MiB, writes mib MiB
    torch.cuda.synchronize()
    print("copied %d MiB x %d (read %d bytes, wrote %d bytes per kernel)" % (mib, reps, n * 4, n * 4))


if __name__ == "__main__":
    main()
