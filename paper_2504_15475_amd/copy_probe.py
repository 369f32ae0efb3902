"""A plain device-to-device copy of known size, for calibrating HBM byte counters.

Run under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE): the copy kernel reads and writes exactly `--mib` MiB, so
the ratio of its counter value to that size is the scale to apply to the same counter read for the race kernel.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--reps", type=int, default=3)
    a = ap.parse_args()
    n = a.mib * (1 << 20) // 4
    src = torch.arange(n, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(a.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {a.mib} MiB x {a.reps} (each copy reads {a.mib} MiB and writes {a.mib} MiB)")


if __name__ == "__main__":
    main()
