"""Plain device-to-device copy of a known size, for scaling HBM traffic counters.

Run under ``rocprofv3 --pmc FETCH_SIZE`` (or ``WRITE_SIZE``): the copy kernel moves exactly
``--mib`` MiB in and the same amount out per launch, so the ratio of the known size to what
the counter reports for it is the factor by which the same counter's readings for the
library's kernels are scaled.  Uses torch only for memory and the copy kernel.
"""
import argparse

import torch


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=512)
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    n = args.mib << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    src.fill_(3)
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    for _ in range(args.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("copied %d MiB x %d" % (args.mib, args.reps))


if __name__ == "__main__":
    main()
