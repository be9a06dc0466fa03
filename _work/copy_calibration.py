"""A plain device-to-device copy of known size, for calibrating HBM traffic counters.

    rocprofv3 --pmc FETCH_SIZE -- python3 paper_2410_03348_amd/copy_calibration.py [--mib 1024] [--reps 5]

The copy kernel reads `mib` MiB and writes `mib` MiB per repetition; the ratio between what a counter reports
for it and that known size is the factor applied to the same counter's reading for the library's kernels.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    n = args.mib * (1 << 20) // 4
    src = torch.full((n,), 1.0, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(args.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("copied %d MiB x %d" % (args.mib, args.reps))


if __name__ == "__main__":
    main()
