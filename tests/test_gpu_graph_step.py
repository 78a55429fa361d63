"""GPU parity of adagc_step_graph: the step whose hyper-parameters and step number are read on the device,
eagerly and as a HIP graph recorded once and replayed for later steps, against the CPU oracle."""
import ctypes
import math

import numpy as np
import pytest
import torch

from paper_2502_11034_amd import binding as B
from paper_2502_11034_amd import workloads as W
from paper_2502_11034_amd.workloads import to_numpy
import parity as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def _workload(lion=False):
    specs = W.llama_like_list(1, 128, 4, 2, 448, 1000) + W.ragged_stress_list(12, 1 << 15, None)
    spikes = {4: (np.arange(0, len(specs), 2), 40.0), 6: (np.arange(1, len(specs), 3), 40.0)}
    return W.Workload(specs, spikes=spikes, bf16_copy=True, grad_dtype=torch.bfloat16 if lion else torch.float32)


def _set(sp, hp, step):
    sp.copy_(torch.frombuffer(bytearray(B.step_params_bytes(hp, step)), dtype=torch.uint8))


def _lockstep_check(run, hp, step, grads, name, warm):
    """Oracle step from the device's pre-step state (mirrored by the caller), then compare everything."""
    norms, coefs, flags = run.ctx.get_norms()
    ref_norms, ref_coefs, ref_flags, thr = run.oracle_step([to_numpy(g) for g in grads], hp, step)
    P.check_scalars("%s step %d" % (name, step), norms, coefs, flags, to_numpy(run.gamma), ref_norms, ref_coefs,
                    ref_flags, run.h_gamma, None if (warm or hp.clip_mode != B.ADAGC_MODE_ADAGC) else thr)
    return ref_flags


def _mirror(run):
    run.h_params = [to_numpy(t) for t in run.params]
    run.h_m = [to_numpy(t) for t in run.m]
    if run.v is not None:
        run.h_v = [to_numpy(t) for t in run.v]
    run.h_gamma = to_numpy(run.gamma)


@pytest.mark.parametrize("optimizer", ["adamw", "lion"])
def test_device_scalars_step_matches_oracle_eagerly(optimizer):
    lion = optimizer == "lion"
    w = _workload(lion)
    run = P.Run(w, optimizer=optimizer)
    model_norm = math.sqrt(sum(float(s) ** 2 * k for s, k in zip(w.sigma, w.numels)))
    hp = B.make_hyper(lr=1e-4 if lion else 3e-4, beta2=0.99 if lion else 0.95, t_start=2, lambda_abs=0.5 * model_norm)
    sp = torch.zeros(ctypes.sizeof(B.adagc_step_params), dtype=torch.uint8, device=DEV)
    for step in range(1, 8):
        grads = w.make_grads(step, DEV)
        _mirror(run)
        m_before = [x.copy() for x in run.h_m]
        _set(sp, hp, step)
        run.ctx.step_graph(run.params, grads, run.m, run.v, run.gamma, sp)
        ref_flags = _lockstep_check(run, hp, step, grads, "device-scalars-" + optimizer, step <= 2)
        exempt = None
        if lion:
            coefs = run.ctx.get_norms()[1].astype(np.float64)
            exempt = [run.lion_exempt(i, to_numpy(grads[i]), m_before[i], coefs[i], hp) for i in range(w.n_tensors)]
        differ = run.compare_state("device-scalars-%s step %d" % (optimizer, step), exempt)
        say("device-scalars-%s step %d: %d values not bit-identical, %d clipped" % (optimizer, step, differ,
                                                                                    int(ref_flags.sum())))
        assert differ <= 4


@pytest.mark.parametrize("mode", [B.ADAGC_MODE_ADAGC, B.ADAGC_MODE_GLOBAL_ADAGC, B.ADAGC_MODE_ZCLIP])
def test_graph_recorded_once_replays_for_later_steps(mode):
    """One eager step, then the step is captured into a graph ONCE (at a warm-up step) and replayed for steps
    3..9 with new gradients, a changing learning rate and the step number all updated in device memory between
    replays; the run crosses from the warm-up branch to the per-tensor rule inside the same recorded graph.
    Every replay is compared with the oracle; eager copies, host read-backs and synchronisations sit between
    the replays."""
    w = _workload()
    run = P.Run(w)
    model_norm = math.sqrt(sum(float(s) ** 2 * k for s, k in zip(w.sigma, w.numels)))
    def hyper(step):
        return B.make_hyper(lr=3e-4 * (1.0 - 0.05 * step), t_start=3, lambda_abs=2.0 * model_norm, clip_mode=mode,
                            ema_beta=0.97 if mode == B.ADAGC_MODE_ZCLIP else 0.99)
    sp = torch.zeros(ctypes.sizeof(B.adagc_step_params), dtype=torch.uint8, device=DEV)
    grads = w.make_grads(1, DEV)                       # static buffers: refilled in place before every step
    name = "graph-mode%d" % mode

    def refill(step):
        for i, g in enumerate(grads):
            w.fill_grad(g, i, step)

    # steps 1 and 2 eagerly (this also uploads the pointer table the recorded launches will use)
    for step in (1, 2):
        refill(step)
        _mirror(run)
        _set(sp, hyper(step), step)
        run.ctx.step_graph(run.params, grads, run.m, run.v, run.gamma, sp)
        _lockstep_check(run, hyper(step), step, grads, name, True)
        run.compare_state("%s step %d" % (name, step))

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    before = [t.clone() for t in run.params + run.m + run.v + [run.gamma]]
    with torch.cuda.graph(graph, stream=side):
        run.ctx.step_graph(run.params, grads, run.m, run.v, run.gamma, sp,
                           stream=torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for x, y in zip(before, run.params + run.m + run.v + [run.gamma]):
        assert torch.equal(x, y)                       # recording runs nothing

    clipped, counts = 0, []
    for step in range(3, 10):
        refill(step)
        _mirror(run)
        _set(sp, hyper(step), step)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref_flags = _lockstep_check(run, hyper(step), step, grads, name, step <= 3)
        differ = run.compare_state("%s step %d" % (name, step))
        say("%s replay for step %d: %d values not bit-identical, %d clipped" % (name, step, differ, int(ref_flags.sum())))
        assert differ <= 4
        clipped += int(ref_flags.sum())
        counts.append(int(ref_flags.sum()))
    assert clipped > 0 and (mode != B.ADAGC_MODE_ADAGC or len(set(counts)) > 1)


def test_device_side_validation_and_capture_rules():
    w = _workload()
    run = P.Run(w, mirror=False)
    hp = B.make_hyper()
    sp = torch.zeros(ctypes.sizeof(B.adagc_step_params), dtype=torch.uint8, device=DEV)
    grads = w.make_grads(1, DEV)
    _set(sp, hp, 1)
    run.ctx.step_graph(run.params, grads, run.m, run.v, run.gamma, sp)
    run.ctx.get_norms()
    before = [t.clone() for t in run.params + run.m + run.v + run.copies + [run.gamma]]

    def code(f):
        try:
            f()
        except B.AdagcError as e:
            return e.code
        return B.ADAGC_OK

    # parameters the host entry point would reject: nothing changes, the read-back reports it
    for bad, step in ((B.make_hyper(beta1=1.5), 2), (B.make_hyper(lambda_abs=0.0), 2), (B.make_hyper(), 0),
                      (B.make_hyper(clip_mode=7), 2), (B.make_hyper(lr=float("nan")), 2)):
        _set(sp, bad, step)
        run.ctx.step_graph(run.params, grads, run.m, run.v, run.gamma, sp)
        assert code(run.ctx.get_norms) == B.ADAGC_ERR_INVALID_ARG
        for x, y in zip(before, run.params + run.m + run.v + run.copies + [run.gamma]):
            assert torch.equal(x, y)
    # a valid step afterwards works, and an ordinary step clears the report
    _set(sp, hp, 2)
    run.ctx.step_graph(run.params, grads, run.m, run.v, run.gamma, sp)
    assert code(run.ctx.get_norms) == B.ADAGC_OK
    assert not torch.equal(before[0], run.params[0])
    _set(sp, B.make_hyper(beta2=-1.0), 3)
    run.ctx.step_graph(run.params, grads, run.m, run.v, run.gamma, sp)
    assert code(run.ctx.get_norms) == B.ADAGC_ERR_INVALID_ARG
    run.ctx.step(run.params, grads, run.m, run.v, run.gamma, hp, 3)
    assert code(run.ctx.get_norms) == B.ADAGC_OK

    # while capturing: other tensor pointers than the previous call's, or active profiling, are refused
    other = [g.clone() for g in grads]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    codes = []
    with torch.cuda.graph(graph, stream=side):
        s = torch.cuda.current_stream().cuda_stream
        codes.append(code(lambda: run.ctx.step_graph(run.params, other, run.m, run.v, run.gamma, sp, stream=s)))
        run.ctx.step_graph(run.params, grads, run.m, run.v, run.gamma, sp, stream=s)
    assert codes == [B.ADAGC_ERR_STATE]
    _set(sp, hp, 4)
    torch.cuda.synchronize()
    snapshot = run.params[0].clone()
    graph.replay()
    torch.cuda.synchronize()
    assert not torch.equal(snapshot, run.params[0])
    assert code(run.ctx.get_norms) == B.ADAGC_OK
