"""Plain device-to-device copy of a known size, used to calibrate the HBM byte counters
(FETCH_SIZE / WRITE_SIZE) that rocprofv3 reads for the chain kernels:

    rocprofv3 --pmc FETCH_SIZE -- python3 -m paper_1708_04801_amd.copy_probe

copies `--mib` MiB (default 1024) `--reps` times with torch's copy kernel; every dispatch reads
and writes exactly that many bytes, so counter value / bytes gives the counter's unit.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args()
    n = args.mib * (1 << 20) // 4
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(args.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {args.mib} MiB x {args.reps}: each dispatch reads and writes {n * 4} bytes")


if __name__ == "__main__":
    main()
