"""Benchmark of the fused AdaGC + AdamW step on Llama-3-8B-shaped synthetic tensors, one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config1|config2|config3|config4|config5]

A "step" is one pass of the whole hot path (segmented norms, per-tensor clip rule + EMA, fused
clip + optimizer update) over the full parameter list, inputs resident in HBM.  Prints ONE JSON
line: throughput as effective GB/s under the two-pass algorithmic byte count, ms per step, the
roofline record of the dominant kernel (measured with HIP events on the step's stream), and the
CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth


def algorithmic_bytes(workload_name):
    """Bytes per parameter that the method itself must move: the norm pass reads g once (the norm of a
    tensor must be complete before any of its elements is updated, Eq. 3); the update pass reads
    g, theta, m(, v) and writes theta, m(, v)(, bf16 copy)."""
    table = {
        # name: (norm read, update read, update write)
        "config1": (4, 16, 12),     # fp32 everything, no copy (launch-bound: 17 MB per step)
        "config2": (4, 16, 12),     # fp32 everything, no copy
        "config3": (4, 16, 14),     # + bf16 copy
        "config4": (2, 10, 10),     # Lion: bf16 g; theta, m fp32; + bf16 copy
        "config5": (4, 16, 12),
    }
    return table[workload_name]


def kernel_source_hash():
    h = hashlib.sha256()
    for name in ("kernels.hip", "adagc_internal.h"):
        with open(os.path.join(ROOT, "paper_2502_11034_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload_name, kernel):
    """HBM bytes per launch from stored rocprofv3 --pmc runs, or None if the kernel source has
    changed since they were taken (profiles/hbm_traffic.json is written by hand from those runs)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    if rec.get("kernel_source_hash") != kernel_source_hash():
        return None
    return rec.get(workload_name, {}).get(kernel)


def cpu_baseline(workload_name, budget_seconds=20.0):
    """Time the CPU oracle, as it stands, on a bounded sample of the same workload, drawn by the workload's
    own generator: the all-cores build (the same source with OpenMP) on every thread the host gives this
    process, and the one-thread definition beside it on a smaller part of the same sample."""
    import numpy as np
    import oracle
    from paper_2502_11034_amd import workloads as W
    from paper_2502_11034_amd.workloads import to_numpy

    w = {"config1": W.config1, "config2": W.config2, "config3": W.config3, "config4": W.config4,
         "config5": W.config5}[workload_name]()
    if workload_name in ("config3", "config4"):
        picked = [i for i, s in enumerate(w.specs) if s.name.startswith("l0.") or s.name in ("embed", "final_norm")]
        sample = "embedding, layer 0 and final norm of the Llama-3-8B-shaped list"
    elif workload_name == "config5":
        picked = list(range(0, 20000, 25)) + [20000]
        sample = "every 25th tensor of the ragged list and its 128256x4096 tensor"
    else:
        picked = list(range(w.n_tensors))
        sample = "the whole list"
    lion = workload_name == "config4"
    hp = (oracle.Hyper(lr=1e-4, beta1=0.9, beta2=0.99, optimizer=oracle.LION, grad_dtype=oracle.GRAD_BF16) if lion
          else oracle.Hyper())
    rd, ur, uw = algorithmic_bytes(workload_name)

    def state(idx):
        theta = [to_numpy(w.init_param(i, "cpu")) for i in idx]
        m = [np.zeros(w.numels[i], np.float32) for i in idx]
        v = None if lion else [np.zeros(w.numels[i], np.float32) for i in idx]
        copies = [np.zeros(w.numels[i], np.uint16) for i in idx] if w.bf16_copy else None
        return theta, m, v, copies, np.zeros(len(idx), np.float32)

    def timed(idx, grads_by_step, limit):
        theta, m, v, copies, gamma = state(idx)
        n = sum(w.numels[i] for i in idx)
        steps, elapsed = 0, 0.0
        while steps < len(grads_by_step) and (steps < 2 or elapsed < limit):
            t0 = time.perf_counter()
            oracle.adagc_step(theta, grads_by_step[steps], m, v, gamma, hp, steps + 1, copies)
            elapsed += time.perf_counter() - t0
            steps += 1
        return {"gbps": (rd + ur + uw) * n * steps / elapsed / 1e9, "ns_per_param_step": elapsed / steps / n * 1e9,
                "steps": steps, "seconds": elapsed, "params": n, "tensors": len(idx)}

    max_steps = 5 if workload_name in ("config3", "config4", "config5") else 10
    grads = [[to_numpy(w.make_grad(i, t, "cpu")) for i in picked] for t in range(1, 4)]    # steps 1..3 (3 = spike step)
    grads = (grads * max_steps)[:max_steps]
    with oracle.all_cores():
        threads = oracle.num_threads()
        many = timed(picked, grads, 0.6 * budget_seconds)
    # the one-thread definition on the first tensors of the sample that hold about a quarter of it
    # (a tensor that is more than half of the sample is left to the all-cores run)
    part, acc = [], 0
    for k, i in enumerate(picked):
        if len(picked) > 1 and w.numels[i] > 0.5 * many["params"]:
            continue
        part.append(k)
        acc += w.numels[i]
        if acc >= 0.25 * many["params"]:
            break
    one = timed([picked[k] for k in part], [[g[k] for k in part] for g in grads], 0.4 * budget_seconds)
    return {"value": round(many["gbps"], 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "host_cpus": os.cpu_count(),
            "sample": "%s (%d tensors, %d params) from the workload's own generator, %d steps in %.1f s on %d threads, "
                      "%.2f ns/param/step" % (sample, many["tensors"], many["params"], many["steps"], many["seconds"],
                                               threads, many["ns_per_param_step"]),
            "one_thread": {"value": round(one["gbps"], 3), "unit": "GB/s", "cores": 1,
                           "sample": "%d tensors of the same sample (%d params), %d steps in %.1f s, %.2f ns/param/step"
                                     % (one["tensors"], one["params"], one["steps"], one["seconds"],
                                        one["ns_per_param_step"])}}


SCHEDULE_LEN = {"config1": 20, "config2": 10, "config3": 5, "config4": 5, "config5": 10}   # steps each workload states


def placement_probe(args):
    """The same benchmark in a child process whose arrays are allocated in the order known to be slow
    (params, m, v, copies, then gradients): where the driver puts the arrays physically changes the
    update kernel's time, and this shows the far end of that spread.  Must run before this process
    touches the GPU (the two workloads do not fit side by side)."""
    import subprocess
    cmd = [sys.executable, os.path.abspath(__file__), "--workload", args.workload, "--steps", str(min(args.steps, 5)),
           "--warmup", "3", "--alloc-order", "slow", "--no-cpu-baseline", "--no-placement-probe"]
    try:
        res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
        line = [l for l in res.stdout.splitlines() if l.startswith("{")][-1]
        rec = json.loads(line)
        return {"alloc_order": "params, m, v, copies, gradients", "ms_per_step": rec["ms_per_step"],
                "update_ms": rec["kernels_ms"]["update"], "steps": rec["steps"]}
    except Exception as exc:            # the probe is extra information; the benchmark itself goes on
        return {"error": "%s: %s" % (type(exc).__name__, exc)}


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix-core rate


def muon_bench(args):
    """Muon with AdaGC on the 224 hidden matrices of the Llama-3-8B-shaped list (q, k, v, o, gate, up, down of every
    layer: the tensors Muon is used for; embeddings, head and norm weights stay with AdamW).  Another roofline than the
    headline workload: the step is bound by the Newton-Schulz products on the matrix cores."""
    import numpy as np
    import torch
    from paper_2502_11034_amd import binding as B
    from paper_2502_11034_amd import workloads as W

    dev = "cuda:0"
    torch.cuda.set_device(0)
    specs = [s for s in W.llama3_8b_list() if len(s.shape) == 2 and "." in s.name]        # l<k>.q, l<k>.gate, ...
    w = W.Workload(specs)
    shapes = [s.shape for s in specs]
    grads = {p: w.make_grads(p, dev) for p in (1, 2)}
    params, mom, _, _ = w.make_state(dev, "lion")
    gamma = torch.zeros(w.n_tensors, dtype=torch.float32, device=dev)
    ctx = B.AdaGC(w.numels, B.ADAGC_OPT_MUON, B.ADAGC_GRAD_F32)
    ctx.muon_attach(shapes)
    hp = B.make_hyper(lr=0.02, weight_decay=0.1, t_start=1)
    mh = B.make_muon_hyper()
    p_ptr, m_ptr = B.ptr_array(params), B.ptr_array(mom)
    g_ptr = {p: B.ptr_array(g) for p, g in grads.items()}
    step = 0
    for _ in range(args.warmup):
        step += 1
        ctx.muon_step(p_ptr, g_ptr[1 + step % 2], m_ptr, gamma, hp, mh, step)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    ctx.profile_begin(args.steps)
    t0 = time.perf_counter()
    for k in range(args.steps):
        step += 1
        ev[k][0].record()
        ctx.muon_step(p_ptr, g_ptr[1 + step % 2], m_ptr, gamma, hp, mh, step)
        ev[k][1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_kernel = ctx.profile_end()                 # [steps, 3] ms: gradient norms, rule, momentum + Newton-Schulz + update
    step_ms = np.array([a.elapsed_time(b) for a, b in ev], dtype=np.float64)
    # Multiply-adds of the iteration.  "full": the three products of a step written out, 4 m^2 n + 2 m^3.  "performed":
    # A = X X^T and A A are symmetric and only their tiles on and below the diagonal are computed (128 x 128 tiles).
    flops, performed = 0.0, 0.0
    for r, c in shapes:
        m, n = min(r, c), max(r, c)
        flops += mh.ns_steps * (4.0 * m * m * n + 2.0 * m * m * m)
        half = (m * m + 128.0 * m) / 2.0                       # elements of the lower triangle of tiles
        performed += mh.ns_steps * (2.0 * half * n + 2.0 * half * m + 2.0 * m * m * n)
    ms = float(np.median(step_ms))
    ns_ms = float(per_kernel[:, 2].mean())
    out = {
        "metric": "Muon+AdaGC step: Newton-Schulz TFLOP/s (multiplications performed) over the whole step, hidden matrices of Llama-3-8B shapes",
        "value": round(performed / (ms * 1e-3) / 1e12, 1), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 3), "ms_min": round(float(step_ms.min()), 3), "ms_max": round(float(step_ms.max()), 3),
        "ms_mean_wall_clock": round((t1 - t0) / args.steps * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "muon: %d matrices, %d params, fp32 grads, fp32 theta and momentum, bf16 Newton-Schulz (%d steps)"
                               % (w.n_tensors, w.total_params, mh.ns_steps),
                   "flops_per_step_performed": performed, "flops_per_step_full_products": flops,
                   "tflops_full_product_equivalent": round(flops / (ms * 1e-3) / 1e12, 1)},
        "kernels_ms": {"sumsq_partials": round(float(per_kernel[:, 0].mean()), 4), "finalize": round(float(per_kernel[:, 1].mean()), 4),
                       "momentum_newton_schulz_update": round(ns_ms, 3)},
        "roofline": {"kernel": "gemm_nt_bf16_kernel (with the elementwise kernels between its launches)", "bound": "mfma",
                     "achieved": round(performed / (ns_ms * 1e-3) / 1e12, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(performed / (ns_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None},
    }
    ctx.close()
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config3", choices=["config1", "config2", "config3", "config4", "config5", "muon"])
    ap.add_argument("--grid-blocks", type=int, default=0, help="launch tuning: workgroups of the persistent grids")
    ap.add_argument("--unroll", type=int, default=0, help="launch tuning: vectors in flight per lane per stream")
    ap.add_argument("--nontemporal", type=int, default=0, help="launch tuning: 1 on, 2 off")
    ap.add_argument("--schedule", type=int, default=0, help="launch tuning: parts of the visiting order")
    ap.add_argument("--schedule-run", type=int, default=0, help="launch tuning: chunks an XCD takes in a row")
    ap.add_argument("--update-split", type=int, default=0, help="launch tuning: work items of the update kernel per chunk")
    ap.add_argument("--telemetry", action="store_true", help="also reduce per-tensor |m|, |v|, |update| norms")
    ap.add_argument("--clip-mode", type=int, default=0,
                    help="0 AdaGC (default), 1 GlobalGC, 2 Global AdaGC, 3 ZClip, 4 AGC, 5 Clippy (the paper's settings for each)")
    ap.add_argument("--t-start", type=int, default=1, help="warm-up steps (1 = only the initialising step)")
    ap.add_argument("--alloc-order", default="good", choices=["good", "slow"],
                    help="good: one gradient batch, params, m, v, copies, other gradient batches; slow: params, m, v, copies, gradients")
    ap.add_argument("--no-placement-probe", action="store_true",
                    help="skip the child process that measures the slow allocation order")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on exactly one GPU (no sharding, no collectives); use --gpus 1")

    if args.workload == "muon":
        return muon_bench(args)
    worst = None
    if not args.no_placement_probe and args.alloc_order == "good":
        worst = placement_probe(args)          # before anything here touches the GPU

    import numpy as np
    import torch
    from paper_2502_11034_amd import binding as B
    from paper_2502_11034_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    dev = "cuda:0"
    torch.cuda.set_device(0)

    w = {"config1": W.config1, "config2": W.config2, "config3": W.config3, "config4": W.config4, "config5": W.config5}[args.workload]()
    lion = args.workload == "config4"
    optimizer = B.ADAGC_OPT_LION if lion else B.ADAGC_OPT_ADAMW
    grad_dtype = B.ADAGC_GRAD_BF16 if w.grad_dtype == torch.bfloat16 else B.ADAGC_GRAD_F32
    rule = dict(t_start=args.t_start, clip_mode=args.clip_mode,
                lambda_abs=1.0 if (args.clip_mode or args.t_start > 1) else float("inf"))
    if args.clip_mode == 3:
        rule.update(ema_beta=0.97, z_thres=2.0)            # appendix "Clipping Hyper-Parameters"
    elif args.clip_mode == 4:
        rule.update(lambda_rel=1e-3)
    elif args.clip_mode == 5:
        rule.update(lambda_rel=1e-2, lambda_abs=0.5)
    update_clip = args.clip_mode in (4, 5)
    hp = (B.make_hyper(lr=1e-4, beta1=0.9, beta2=0.99, weight_decay=0.1, **rule) if lion else B.make_hyper(**rule))

    # Gradient batches, resident: the workload's own generator and spike schedule.  Step t of the run
    # presents position p = (t-1) mod L + 1 of the workload's L-step schedule: the batch of that spike
    # step if p is one, else one of two ordinary batches in turn.  (Real gradients differ on every step;
    # two ordinary batches already give small tensors their natural clip rate, large tensors clip on
    # spikes only.)
    sched_len = SCHEDULE_LEN[args.workload]
    batch_steps = [1, 2] + sorted(p for p in w.spikes if p <= sched_len)

    def batch_of(t):
        p = (t - 1) % sched_len + 1
        return p if p in w.spikes else (1 if t % 2 else 2)

    # Allocation order.  Where the driver puts the arrays physically changes the update kernel's time
    # by up to ~8 % (measured: the position of theta, m, v and the copies matters, that of the gradients
    # does not).  "good": one gradient batch, then params, m, v, copies, then the other gradient batches
    # (update 37.4 ms in the first process of a fresh machine, where memory is handed out linearly, and
    # 38.0-38.4 ms in later processes); "slow", measured by the child process above: state first.
    if args.alloc_order == "good":
        grads = {batch_steps[0]: w.make_grads(batch_steps[0], dev)}
        params, m, v, copies = w.make_state(dev, "lion" if lion else "adamw")
        for p in batch_steps[1:]:
            grads[p] = w.make_grads(p, dev)
    else:
        params, m, v, copies = w.make_state(dev, "lion" if lion else "adamw")
        grads = {p: w.make_grads(p, dev) for p in batch_steps}
    gamma = torch.zeros(w.n_tensors, dtype=torch.float32, device=dev)
    ctx = B.AdaGC(w.numels, optimizer, grad_dtype, w.bf16_copy, grid_blocks=args.grid_blocks,
                  unroll=args.unroll, nontemporal=args.nontemporal, schedule=args.schedule,
                  telemetry=args.telemetry, update_split=args.update_split,
                  schedule_run=args.schedule_run, update_clipping=update_clip)
    if copies is not None:
        ctx.set_param_copies(copies)
    p_ptr, m_ptr = B.ptr_array(params), B.ptr_array(m)
    v_ptr = B.ptr_array(v) if v is not None else None
    g_ptr = {p: B.ptr_array(g) for p, g in grads.items()}
    stream = torch.cuda.current_stream().cuda_stream

    step = 0
    for _ in range(args.warmup):
        step += 1
        ctx.step(p_ptr, g_ptr[batch_of(step)], m_ptr, v_ptr, gamma, hp, step, stream=stream)
    torch.cuda.synchronize()

    # Timed region: exactly --steps steps between two synchronisations; each step also sits between two
    # events on the stream it is enqueued on, and the library records its own per-kernel events.
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    clipped_per_step = []
    ctx.profile_begin(args.steps)
    t0 = time.perf_counter()
    for k in range(args.steps):
        step += 1
        ev[k][0].record()
        ctx.step(p_ptr, g_ptr[batch_of(step)], m_ptr, v_ptr, gamma, hp, step, stream=stream)
        ev[k][1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_kernel = ctx.profile_end()                 # [steps, 3] ms: norm, finalize, update
    norms, coefs, flags = ctx.get_norms()
    step_ms = np.array([a.elapsed_time(b) for a, b in ev], dtype=np.float64)

    n = w.total_params
    rd, ur, uw = algorithmic_bytes(args.workload)
    if update_clip:
        rd = ur                # the first pass reads g, theta, m, v for the direction's norms instead of g alone
    ms_per_step = float(np.median(step_ms))
    ms_wall_mean = (t1 - t0) / args.steps * 1e3
    bytes_two_pass = (rd + ur + uw) * n
    bytes_once = (ur + uw) * n
    value = bytes_two_pass / (ms_per_step * 1e-3) / 1e9
    k_norm, k_fin, k_upd = (float(per_kernel[:, j].mean()) for j in range(3))
    upd_bytes = (ur + uw) * n
    upd_gbps = upd_bytes / (k_upd * 1e-3) / 1e9
    norm_gbps = rd * n / (k_norm * 1e-3) / 1e9

    out = {
        "metric": "fused AdaGC+%s step: effective GB/s (two-pass algorithmic bytes), %s" % (
            "Lion" if lion else "AdamW",
            {"config1": "tiny 2-layer transformer shapes", "config2": "GPT-2-small shapes", "config3": "Llama-3-8B shapes", "config4": "Llama-3-8B shapes",
             "config5": "ragged stress list"}[args.workload]),
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_min": round(float(step_ms.min()), 4),
        "ms_max": round(float(step_ms.max()), 4),
        "ms_mean_wall_clock": round(ms_wall_mean, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": "%s: %d tensors, %d params, %s grads, %s%s" % (
            args.workload, w.n_tensors, n, "bf16" if grad_dtype else "fp32",
            "Lion fp32 theta/m" if lion else "AdamW fp32 theta/m/v", ", bf16 param copy" if w.bf16_copy else ""),
            "bytes_per_param_two_pass": rd + ur + uw, "bytes_per_param_each_array_once": ur + uw,
            "clip_mode": args.clip_mode, "t_start": args.t_start, "telemetry": bool(args.telemetry),
            "alloc_order": args.alloc_order,
            "gradient_batches": "steps %s of the workload's generator, presented by its %d-step spike schedule"
                                % (batch_steps, sched_len)},
        "ms_per_step_is": "median of the per-step event times",
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "pct_hbm_peak_each_array_once": round(100.0 * bytes_once / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
        "effective_gbps_each_array_once": round(bytes_once / (ms_per_step * 1e-3) / 1e9, 1),
        "kernels_ms": {"sumsq_partials": round(k_norm, 4), "finalize": round(k_fin, 4), "update": round(k_upd, 4),
                       "update_median": round(float(np.median(per_kernel[:, 2])), 4),
                       "update_min": round(float(per_kernel[:, 2].min()), 4),
                       "update_max": round(float(per_kernel[:, 2].max()), 4)},
        "norm_kernel_gbps": round(norm_gbps, 1),
        "tensors_clipped_last_step": int(flags.sum()),
        "roofline": {"kernel": "update_kernel", "bound": "hbm", "achieved": round(upd_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(upd_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": measured_traffic(args.workload, "update_kernel")},
    }
    if worst is not None:
        out["placement_worst"] = worst
        out["placement_worst_ms"] = worst.get("ms_per_step")
    ctx.close()
    del params, m, v, copies, grads
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
