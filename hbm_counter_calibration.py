"""Plain device-to-device copy of known size, for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters.

Run under ``rocprofv3 --pmc FETCH_SIZE`` (then ``WRITE_SIZE``): the copy kernel of each iteration reads
exactly ``--mib`` MiB and writes exactly ``--mib`` MiB, so (counter value in KiB per dispatch) / (MiB * 1024)
is the factor by which the counter over- or under-reports HBM traffic on this machine.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--iters", type=int, default=5)
    args = ap.parse_args()
    n = args.mib * (1 << 20) // 2
    src = torch.ones(n, dtype=torch.bfloat16, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(args.iters):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("copied %d MiB x %d" % (args.mib, args.iters))


if __name__ == "__main__":
    main()
