"""Plain device-to-device copy of a known size, for calibrating hardware counters.

Run under `rocprofv3 --pmc FETCH_SIZE` (then `WRITE_SIZE`): the copy kernel reads and writes
exactly `--mib` MiB per launch, so the ratio of the counter's reading to that figure is the
scale factor to apply to the same counter's reading for the library's kernels.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=2048)
    ap.add_argument("--launches", type=int, default=3)
    args = ap.parse_args()
    n = args.mib * 1024 * 1024 // 4
    src = torch.empty(n, dtype=torch.float32, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(args.launches):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("copied %d MiB x %d launches" % (args.mib, args.launches))


if __name__ == "__main__":
    main()
