"""What the memory system gives a kernel shaped like the update kernel, for several read : write mixes.

Measurement tool (like copy_calibration.py), not part of the library: it loads libadagc_probe.so, built from
csrc/memory_probe.hip, and times one streaming kernel per mix with HIP events.  The figures put the update kernel's
own rate (4 arrays read, 3 of them written in place, plus a bf16 copy) beside what the same access shape reaches when
it only reads, only writes, or does both:

    python3 -m paper_2502_11034_amd.memory_probe [--gib-per-array 16] [--gap-gib 0]
"""
import argparse
import ctypes
import os

import torch

from . import build as _build

PROBE_LIB = os.path.join(_build.HERE, "libadagc_probe.so")
MIXES = [(1, 0), (4, 0), (0, 1), (0, 4), (1, 1), (2, 1), (4, 3)]


def lib():
    if not os.path.exists(PROBE_LIB):
        _build.build_probe()
    L = ctypes.CDLL(PROBE_LIB)
    L.adagc_probe_stream.restype = ctypes.c_int
    L.adagc_probe_stream.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_void_p]
    return L


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gib-per-array", type=float, default=16.0)
    ap.add_argument("--gap-gib", type=float, default=0.0, help="unused memory allocated between two arrays (their distance matters)")
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    L = lib()
    elems = int(args.gib_per_array * (1 << 30) / 4) // 4096 * 4096
    arrays, gaps = [], []
    for _ in range(4):
        arrays.append(torch.zeros(elems, dtype=torch.float32, device="cuda:0"))
        if args.gap_gib > 0:
            gaps.append(torch.empty(int(args.gap_gib * (1 << 30)), dtype=torch.uint8, device="cuda:0"))
    ptrs = (ctypes.c_void_p * 4)(*[a.data_ptr() for a in arrays])
    print("arrays: 4 x %.1f GiB fp32, %s between them; first addresses %s" % (
        args.gib_per_array, "%.1f GiB" % args.gap_gib if args.gap_gib else "nothing", ", ".join(hex(a.data_ptr()) for a in arrays)))
    print("%-28s %10s %10s" % ("arrays read : written", "ms", "TB/s"))
    for nr, nw in MIXES:
        def run():
            rc = L.adagc_probe_stream(ptrs, nr, nw, elems, None)
            if rc != 0:
                raise RuntimeError("adagc_probe_stream failed")
        run()
        torch.cuda.synchronize()
        times = []
        for _ in range(args.reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            run()
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        ms = sorted(times)[len(times) // 2]
        nbytes = (nr + nw) * elems * 4
        print("%-28s %10.3f %10.2f" % ("%d : %d%s" % (nr, nw, " (in place)" if nr and nw else ""), ms, nbytes / ms / 1e9), flush=True)


if __name__ == "__main__":
    main()
