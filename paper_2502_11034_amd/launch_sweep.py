"""Time the step under different launch settings on one resident workload.

    python -m paper_2502_11034_amd.launch_sweep [--workload config3] [--steps 4]

The state is allocated once, so that every setting runs on the same physical placement of the
arrays (placement alone moves the update kernel by 10 % or more between processes); each setting
gets its own context.  Prints one line per setting: ms per step and the three kernel durations
measured with HIP events on the step's stream.  The library's defaults were chosen from this
table on an MI355X; on other parts re-run it and pass the winners through adagc_config.
"""
import argparse
import itertools
import time

import torch

from . import binding as B
from . import workloads as W


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="config3", choices=["config2", "config3", "config4", "config5"])
    ap.add_argument("--steps", type=int, default=4)
    args = ap.parse_args()
    dev = "cuda:0"
    w = getattr(W, args.workload)()
    lion = args.workload == "config4"
    opt = B.ADAGC_OPT_LION if lion else B.ADAGC_OPT_ADAMW
    gd = B.ADAGC_GRAD_BF16 if w.grad_dtype == torch.bfloat16 else B.ADAGC_GRAD_F32
    hp = B.make_hyper(lr=1e-4, beta1=0.9, beta2=0.99) if lion else B.make_hyper()
    grads = w.make_grads(2, dev)
    params, m, v, copies = w.make_state(dev, "lion" if lion else "adamw")
    gamma = torch.zeros(w.n_tensors, dtype=torch.float32, device=dev)
    ptrs = tuple(B.ptr_array(x) if x is not None else None for x in (params, grads, m, v))
    print("%s: %d tensors, %d params" % (args.workload, w.n_tensors, w.total_params), flush=True)

    def run(**kw):
        ctx = B.AdaGC(w.numels, opt, gd, w.bf16_copy, **kw)
        if copies is not None:
            ctx.set_param_copies(copies)
        for s in range(1, 3):
            ctx.step(*ptrs, gamma, hp, s)
        torch.cuda.synchronize()
        ctx.profile_begin(args.steps)
        t0 = time.perf_counter()
        for s in range(3, 3 + args.steps):
            ctx.step(*ptrs, gamma, hp, s)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms = ctx.profile_end().mean(axis=0)
        ctx.close()
        return (t1 - t0) / args.steps * 1e3, ms

    def show(tag, **kw):
        tot, ms = run(**kw)
        print("%-58s step %7.3f ms | norm %6.3f  finalize %5.3f  update %7.3f" % (tag, tot, ms[0], ms[1], ms[2]),
              flush=True)

    show("defaults")
    print("-- workgroups: one work item each (default) against persistent grids")
    for grid in (512, 1024, 2048, 4096):
        show("grid_blocks=%d (persistent, static round-robin)" % grid, grid_blocks=grid)
    print("-- non-temporal hints")
    for nt, name in ((1, "on (default)"), (2, "off")):
        show("nontemporal %s" % name, nontemporal=nt)
    print("-- visiting order: parts x run (XCD x works in part x mod parts; sharing XCDs take runs of chunks in turn)")
    for parts, runlen in ((1, 1), (1, 8), (2, 1), (2, 4), (2, 8), (2, 16), (2, 64), (4, 1), (4, 4), (4, 8), (8, 1), (64, 1),
                       (1021, 1)):
        show("schedule=%d schedule_run=%d%s" % (parts, runlen, " (default)" if (parts, runlen) == (2, 8) else ""),
             schedule=parts, schedule_run=runlen)
    print("-- 128-bit vectors per lane per array in flight")
    for unroll in (1, 2, 4):
        show("unroll=%d%s" % (unroll, " (default)" if unroll == 4 else ""), unroll=unroll)
    print("-- work items of the update kernel per chunk (1 = whole chunks; default 4 = 4096 elements)")
    for split in (1, 2, 4):
        show("update_split=%d" % split, update_split=split)
    show("update_split=16 unroll=1", update_split=16, unroll=1)
    print("-- combinations")
    for grid, nt, parts in itertools.product((0, 1024), (1, 2), (2, 8)):
        show("grid_blocks=%d nontemporal=%d schedule=%d" % (grid, nt, parts), grid_blocks=grid, nontemporal=nt,
             schedule=parts)
    print("-- telemetry")
    show("telemetry=1", telemetry=True)


if __name__ == "__main__":
    main()
