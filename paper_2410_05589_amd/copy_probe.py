"""Calibration for the HBM traffic counters: a plain device-to-device copy of known size.

Run under `rocprofv3 --pmc FETCH_SIZE` (then `--pmc WRITE_SIZE`): the copy kernel reads and
writes exactly `--mib` MiB, so counter / (mib * 1024) is the factor by which the counter (in
KiB) has to be divided for other kernels.  The buffers are larger than the 256 MB Infinity
Cache so the traffic really reaches HBM.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--iters", type=int, default=5)
    args = ap.parse_args()
    n = args.mib * (1 << 20)
    src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    for _ in range(args.iters):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("copied %d MiB x %d" % (args.mib, args.iters))


if __name__ == "__main__":
    main()
