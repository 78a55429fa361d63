"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Sizes here finish in seconds on the oracle and still span many chunks, ragged tails and
tensors smaller than one lane-vector.  Full-size cases are in test_gpu_parity_fullsize.py."""
import ctypes
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2502_11034_amd import binding as B
from paper_2502_11034_amd import workloads as W
from paper_2502_11034_amd.workloads import to_numpy
import parity as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def trajectory(run, hp, steps, name, lockstep=False):
    """Advance device and oracle side by side.  lockstep=True re-seeds the oracle's state from the
    device before every step (strict one-step comparison)."""
    clipped_total = 0
    for step in range(1, steps + 1):
        grads = run.w.make_grads(step, DEV)
        grads_np = [to_numpy(g) for g in grads]
        if lockstep:
            run.h_params = [to_numpy(t) for t in run.params]
            run.h_m = [to_numpy(t) for t in run.m]
            if run.v is not None:
                run.h_v = [to_numpy(t) for t in run.v]
            run.h_gamma = to_numpy(run.gamma)
        m_before = [x.copy() for x in run.h_m] if run.optimizer == B.ADAGC_OPT_LION else None
        norms, coefs, flags = run.gpu_step(grads, hp, step)
        ref_norms, ref_coefs, ref_flags, thr = run.oracle_step(grads_np, hp, step)
        warm = (step - 1) < hp.t_start
        P.check_scalars("%s step %d" % (name, step), norms, coefs, flags, to_numpy(run.gamma),
                        ref_norms, ref_coefs, ref_flags, run.h_gamma,
                        None if (warm or hp.clip_mode != B.ADAGC_MODE_ADAGC) else thr)
        exempt = None
        if run.optimizer == B.ADAGC_OPT_LION:
            update_clip = hp.clip_mode in (B.ADAGC_MODE_AGC, B.ADAGC_MODE_CLIPPY)     # the gradient is not scaled there
            exempt = [run.lion_exempt(i, grads_np[i], m_before[i], 1.0 if update_clip else ref_coefs[i], hp)
                      for i in range(run.w.n_tensors)]
        if lockstep or step == steps or step in run.w.spikes:
            differ = run.compare_state("%s step %d" % (name, step), exempt)
            say("%s step %d: state within relative 1e-5 everywhere (%d values not bit-identical), %d clipped"
                % (name, step, differ, int(ref_flags.sum())))
            # both sides round a double result once: all but a vanishing fraction is bit-identical
            n_values = (3 if run.v is not None else 2) * run.w.total_params
            assert differ <= max(4, n_values // 100000)
        clipped_total += int(ref_flags.sum())
    return clipped_total


# --------------------------------------------------------------------------- segment table on the device

def test_device_segment_table_matches_enumeration():
    numels = [1, 3, 4, 5, 16383, 16384, 16385, 32768, 50000, 2, 100000]
    ctx = B.AdaGC(numels)
    begin, tensor, index = ctx.get_segment_table()
    ref_chunks, ref_begin = oracle.enumerate_chunks(numels, B.adagc_chunk_elems())
    assert begin.tolist() == ref_begin
    assert tensor.tolist() == [c[0] for c in ref_chunks]
    assert (index.astype(np.int64) * B.adagc_chunk_elems()).tolist() == [c[1] for c in ref_chunks]
    assert ctx.num_chunks() == len(ref_chunks)
    ctx.close()


# --------------------------------------------------------------------------- the named workloads

def test_config1_tiny_transformer_20_steps():
    w = W.config1()
    assert w.n_tensors == 27 and w.total_params == 527872
    run = P.Run(w)
    hp = B.make_hyper(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    clipped = trajectory(run, hp, 20, "config1")
    assert clipped >= 6          # the spiked tensors of steps 7 and 13 at least


def test_config2_gpt2_small_10_steps():
    w = W.config2()
    assert w.n_tensors == 148 and w.total_params == 124439808
    run = P.Run(w)
    hp = B.make_hyper()
    clipped = trajectory(run, hp, 10, "config2")
    assert clipped >= 7


def test_config3_shape_scaled_adamw_bf16_copy():
    """Llama-shaped list (GQA, SwiGLU, RMSNorm) at 1/8 width, 2 layers, with the bf16 copy."""
    specs = W.llama_like_list(2, 512, 8, 2, 1792, 16032)
    w = W.config3(specs)
    w.spikes = W.forced_spike_schedule(len(specs), 5, {3}, 3, 50.0)
    run = P.Run(w)
    clipped = trajectory(run, B.make_hyper(), 5, "config3-scaled", lockstep=True)
    assert clipped >= 3


def test_config4_shape_scaled_lion_bf16_grads():
    specs = W.llama_like_list(2, 512, 8, 2, 1792, 16032)
    w = W.config4(specs)
    w.spikes = W.forced_spike_schedule(len(specs), 5, {3}, 3, 50.0)
    run = P.Run(w, optimizer="lion")
    hp = B.make_hyper(lr=1e-4, beta1=0.9, beta2=0.99, weight_decay=0.1)
    clipped = trajectory(run, hp, 5, "config4-scaled", lockstep=True)
    assert clipped >= 3


def test_config4_lion_trajectory_fp32_grads():
    specs = W.gpt2_like_list(2, 128, 512, 1024, 0)
    w = W.Workload(specs, spikes=W.forced_spike_schedule(len(specs), 6, {4}, 3, 100.0))
    run = P.Run(w, optimizer="lion")
    hp = B.make_hyper(lr=1e-4, beta1=0.9, beta2=0.99, weight_decay=0.1)
    trajectory(run, hp, 6, "lion-fp32", lockstep=True)


def test_config5_ragged_stress_scaled():
    """2000 tensors, log-uniform sizes in [1, 2^17], heavy-tailed outliers, plus one larger tensor."""
    specs = W.ragged_stress_list(2000, 1 << 17, (1000, 4099))
    w = W.config5(specs)
    sizes = np.array(w.numels)
    assert (sizes == 1).any() or sizes.min() <= 3
    run = P.Run(w)
    trajectory(run, B.make_hyper(), 4, "config5-scaled")


# --------------------------------------------------------------------------- edges

def _single(numels, grads, gamma0, hp, step, params=None, optimizer="adamw"):
    """One step on hand-made tensors; returns (run, gpu scalars, oracle scalars)."""
    specs = [W.TensorSpec("t%d" % i, (n,), "matrix") for i, n in enumerate(numels)]
    w = W.Workload(specs)
    run = P.Run(w, optimizer=optimizer)
    run.gamma.copy_(torch.tensor(gamma0, dtype=torch.float32))
    run.h_gamma[:] = np.asarray(gamma0, dtype=np.float32)
    g_dev = [torch.tensor(g, dtype=torch.float32, device=DEV) for g in grads]
    got = run.gpu_step(g_dev, hp, step)
    ref = run.oracle_step([np.asarray(g, dtype=np.float32) for g in grads], hp, step)
    return run, got, ref


def test_chunk_boundary_sizes_and_tiny_tensors():
    c = B.adagc_chunk_elems()
    numels = [1, 2, 3, 4, 5, 63, 64, 65, 255, 256, 257, 1023, 1025, c - 1, c, c + 1, 2 * c - 3, 2 * c, 3 * c + 5]
    rng = np.random.default_rng(0)
    grads = [rng.standard_normal(n).astype(np.float32) * 0.01 for n in numels]
    hp = B.make_hyper(t_start=0)
    gamma0 = [float(np.linalg.norm(g)) * (0.5 if i % 2 else 2.0) for i, g in enumerate(grads)]
    run, got, ref = _single(numels, grads, gamma0, hp, 3)
    P.check_scalars("boundary", *got, to_numpy(run.gamma), ref[0], ref[1], ref[2], run.h_gamma, ref[3])
    assert ref[2].sum() == len(numels) // 2
    run.compare_state("boundary")


def test_degenerate_zero_gradient_and_zero_gamma():
    numels = [8, 8, 8, 1]
    grads = [np.zeros(8), np.full(8, 0.5), np.zeros(8), np.array([2.0])]
    gamma0 = [1.0, 0.0, 0.0, 0.0]
    hp = B.make_hyper(t_start=0)
    run, got, ref = _single(numels, grads, gamma0, hp, 2)
    norms, coefs, flags = got
    assert coefs.tolist() == [1.0, 0.0, 1.0, 0.0] and flags.tolist() == [0, 1, 0, 1]
    assert np.array_equal(coefs.astype(np.float64), ref[1]) and np.array_equal(flags, ref[2])
    assert to_numpy(run.gamma).tolist() == run.h_gamma.tolist()
    assert to_numpy(run.gamma)[1] == 0.0 and to_numpy(run.gamma)[3] == 0.0
    run.compare_state("degenerate")


def test_infinite_lambda_rel_is_plain_adamw():
    """With lambda_rel = +inf (and gamma = 0, where the threshold is NaN) nothing is ever clipped
    and the step is plain AdamW: checked against the library optimizer on the GPU."""
    rng = np.random.default_rng(1)
    numels = [1000, 33, 20000]
    hp = B.make_hyper(lr=1e-2, lambda_rel=math.inf, t_start=0)
    specs = [W.TensorSpec("t%d" % i, (n,), "matrix") for i, n in enumerate(numels)]
    run = P.Run(W.Workload(specs), mirror=False)
    tp = [p.clone().requires_grad_(True) for p in run.params]
    opt = torch.optim.AdamW(tp, lr=1e-2, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1, foreach=False)
    for step in range(1, 6):
        grads = [torch.tensor(rng.standard_normal(n), dtype=torch.float32, device=DEV) * 100.0 ** (step % 3 - 1)
                 for n in numels]
        norms, coefs, flags = run.gpu_step(grads, hp, step)
        assert (coefs == 1.0).all() and not flags.any()
        for p, g in zip(tp, grads):
            p.grad = g.clone()
        opt.step()
    for p, q in zip(run.params, tp):
        np.testing.assert_allclose(to_numpy(p), to_numpy(q), rtol=2e-5, atol=2e-7)


def test_unaligned_pointers_take_the_scalar_path():
    """Views that start 1 element into a buffer are 4-byte aligned only."""
    rng = np.random.default_rng(2)
    numels = [5, 1000, 16384 + 7, 40000]
    hp = B.make_hyper(t_start=0)

    def off(n, fill=None, dtype=torch.float32):
        buf = torch.zeros(n + 1, dtype=dtype, device=DEV)
        view = buf[1:]
        if fill is not None:
            view.copy_(torch.as_tensor(fill, dtype=dtype))
        return view

    params = [off(n, rng.standard_normal(n) * 0.02) for n in numels]
    grads = [off(n, rng.standard_normal(n) * 0.1) for n in numels]
    m = [off(n, rng.standard_normal(n) * 0.01) for n in numels]
    v = [off(n, (rng.standard_normal(n) * 0.01) ** 2) for n in numels]
    copies = [off(n, dtype=torch.bfloat16) for n in numels]
    assert all(t.data_ptr() % 16 != 0 for t in params)
    gamma = torch.tensor([0.01, 10.0, 1.0, 100.0], dtype=torch.float32, device=DEV)
    h = [[to_numpy(t) for t in lst] for lst in (params, grads, m, v)]
    h_gamma = to_numpy(gamma)
    h_copies = [np.zeros(n, np.uint16) for n in numels]
    ctx = B.AdaGC(numels, has_bf16_param_copy=True)
    ctx.set_param_copies(copies)
    ctx.step(params, grads, m, v, gamma, hp, 7)
    norms, coefs, flags = ctx.get_norms()
    ohp = P.oracle_hyper(hp, 0, 0)
    rn, rc, rf = oracle.adagc_step(h[0], h[1], h[2], h[3], h_gamma, ohp, 7, h_copies)
    P.check_scalars("unaligned", norms, coefs, flags, to_numpy(gamma), rn, rc, rf, h_gamma)
    assert rf.any() and not rf.all()
    for i in range(len(numels)):
        P.assert_close("unaligned theta %d" % i, to_numpy(params[i]), h[0][i])
        P.assert_close("unaligned m %d" % i, to_numpy(m[i]), h[2][i])
        P.assert_close("unaligned v %d" % i, to_numpy(v[i]), h[3][i])
        P.assert_bf16_copy("unaligned copy %d" % i, to_numpy(copies[i]), to_numpy(params[i]), h[0][i])
    ctx.close()


def test_warmup_branch_global_clip_and_running_min():
    """t_start = 3 with a finite lambda_abs that the global norm exceeds on steps 1 and 3 only."""
    specs = W.gpt2_like_list(1, 64, 256, 300, 0)
    w = W.Workload(specs, sigma_lo=1e-2, sigma_hi=1e-1,
                   spikes={1: (np.arange(len(specs)), 10.0), 3: (np.arange(len(specs)), 10.0)})
    run = P.Run(w)
    g2 = w.make_grads(2, DEV)
    total = math.sqrt(sum(float((g.double() ** 2).sum()) for g in g2))    # an unspiked step
    hp = B.make_hyper(lambda_abs=3.0 * total, t_start=3)
    for step in range(1, 6):
        grads = w.make_grads(step, DEV)
        norms, coefs, flags = run.gpu_step(grads, hp, step)
        rn, rc, rf, thr = run.oracle_step([to_numpy(g) for g in grads], hp, step)
        P.check_scalars("warmup step %d" % step, norms, coefs, flags, to_numpy(run.gamma), rn, rc, rf,
                        run.h_gamma, None if step <= 3 else thr)
        if step in (1, 3):
            assert rf.all() and (rc < 1.0).all() and len(set(rc.tolist())) == 1
        if step == 2:
            assert not rf.any()
    run.compare_state("warmup")


def test_globalgc_mode_every_step():
    """Eq. 2 on every step: one coefficient for the model, no state."""
    specs = W.gpt2_like_list(2, 128, 512, 1024, 0)
    w = W.Workload(specs, sigma_lo=1e-2, sigma_hi=1e-1, spikes={3: (np.arange(0, len(specs), 2), 20.0)})
    run = P.Run(w)
    g2 = w.make_grads(2, DEV)
    total = math.sqrt(sum(float((g.double() ** 2).sum()) for g in g2))
    hp = B.make_hyper(lambda_abs=2.0 * total, t_start=0, clip_mode=B.ADAGC_MODE_GLOBALGC)
    run.gamma.fill_(3.0)
    run.h_gamma[:] = 3.0
    for step in range(1, 6):
        grads = w.make_grads(step, DEV)
        norms, coefs, flags = run.gpu_step(grads, hp, step)
        rn, rc, rf, _ = run.oracle_step([to_numpy(g) for g in grads], hp, step)
        P.check_scalars("globalgc step %d" % step, norms, coefs, flags, to_numpy(run.gamma), rn, rc, rf, run.h_gamma)
        assert len(set(coefs.tolist())) == 1
        assert bool(rf.all()) == (step == 3) and bool(rf.any()) == (step == 3)
    assert (to_numpy(run.gamma) == 3.0).all()
    run.compare_state("globalgc")


def test_global_adagc_mode_single_adaptive_threshold():
    """One gamma for the whole model (kept in ema_norms[0]): warm-up with Eq. 2, then Eq. 3 on the
    model's norm."""
    specs = W.gpt2_like_list(2, 128, 512, 1024, 0)
    every = np.arange(len(specs))
    w = W.Workload(specs, sigma_lo=1e-2, sigma_hi=1e-1, spikes={1: (every, 5.0), 5: (every[::3], 30.0), 8: (every, 0.2)})
    run = P.Run(w)
    g2 = w.make_grads(2, DEV)
    total = math.sqrt(sum(float((g.double() ** 2).sum()) for g in g2))
    hp = B.make_hyper(lambda_abs=2.0 * total, t_start=2, clip_mode=B.ADAGC_MODE_GLOBAL_ADAGC)
    run.gamma[1:].fill_(7.0)
    run.h_gamma[1:] = 7.0
    seen = []
    for step in range(1, 10):
        grads = w.make_grads(step, DEV)
        norms, coefs, flags = run.gpu_step(grads, hp, step)
        rn, rc, rf, _ = run.oracle_step([to_numpy(g) for g in grads], hp, step)
        P.check_scalars("global-adagc step %d" % step, norms, coefs, flags, to_numpy(run.gamma), rn, rc, rf,
                        run.h_gamma)
        assert len(set(coefs.tolist())) == 1 and len(set(flags.tolist())) == 1
        seen.append(int(rf[0]))
    assert seen[0] == 1 and seen[4] == 1 and 0 in seen
    assert (to_numpy(run.gamma)[1:] == 7.0).all()
    run.compare_state("global-adagc")


def test_zclip_mode_z_score_of_the_global_norm():
    """Table 2's ZClip row: three steps that gather the mean and variance of the model's norm under Eq. 2,
    then the z-score rule.  The model's gradient scale wanders by a few per cent and jumps on steps 6 and 11,
    so that clipped and unclipped steps both occur; the state is (mu, var) in ema_norms[0:2]."""
    specs = W.gpt2_like_list(2, 128, 512, 1024, 0)
    every = np.arange(len(specs))
    scale = {1: 1.3, 2: 1.0, 3: 0.9, 4: 1.05, 5: 0.97, 6: 4.0, 7: 1.0, 8: 0.8, 9: 1.02, 10: 0.99, 11: 1.6, 12: 1.0}
    w = W.Workload(specs, sigma_lo=1e-2, sigma_hi=1e-1, spikes={t: (every, f) for t, f in scale.items()})
    run = P.Run(w)
    g2 = w.make_grads(2, DEV)
    total = math.sqrt(sum(float((g.double() ** 2).sum()) for g in g2))
    hp = B.make_hyper(lambda_abs=1.2 * total, t_start=3, clip_mode=B.ADAGC_MODE_ZCLIP, ema_beta=0.97, z_thres=2.0)
    run.gamma[2:].fill_(7.0)
    run.h_gamma[2:] = 7.0
    seen = []
    for step in range(1, 13):
        grads = w.make_grads(step, DEV)
        norms, coefs, flags = run.gpu_step(grads, hp, step)
        rn, rc, rf, _ = run.oracle_step([to_numpy(g) for g in grads], hp, step)
        P.check_scalars("zclip step %d" % step, norms, coefs, flags, to_numpy(run.gamma), rn, rc, rf, run.h_gamma)
        assert len(set(coefs.tolist())) == 1 and len(set(flags.tolist())) == 1
        seen.append(int(rf[0]))
        say("zclip step %2d: h %.6f clipped %d mu %.6f var %.3e" % (step, rc[0], rf[0], run.h_gamma[0], run.h_gamma[1]))
    assert seen[0] == 1 and seen[1] == 0 and seen[5] == 1 and seen[10] == 1 and 0 in seen[3:]
    assert (to_numpy(run.gamma)[2:] == 7.0).all()
    run.compare_state("zclip")
    # the threshold must be positive (NaN and zero rejected before anything is enqueued)
    for bad in (0.0, -1.0, float("nan")):
        with pytest.raises(B.AdagcError) as e:
            run.ctx.step(run.params, grads, run.m, run.v, run.gamma, B.make_hyper(clip_mode=B.ADAGC_MODE_ZCLIP, z_thres=bad), 13)
        assert e.value.code == B.ADAGC_ERR_INVALID_ARG


def _update_clip_workload(lion=False):
    """Matrices (theta ~ 0.02), norm weights (theta = 1) and biases (theta = 0), ragged sizes, several chunks."""
    specs = W.gpt2_like_list(2, 128, 512, 1024, 0) + W.ragged_stress_list(10, 1 << 16, (3 * 16384 + 5,))
    return W.Workload(specs, sigma_lo=1e-3, sigma_hi=1e-1, bf16_copy=True,
                      grad_dtype=torch.bfloat16 if lion else torch.float32)


@pytest.mark.parametrize("optimizer", ["adamw", "lion"])
def test_agc_mode_update_clipping_by_weight_norm(optimizer):
    """Table 2's AGC row: the gradient is left alone, each tensor's direction is scaled by
    min{1, lambda_rel ||theta|| / ||Delta||}.  lambda_rel 20: matrices are clipped (ratio ~0.4), norm weights
    are not (ratio ~20), zero-initialised biases get coefficient 0 and stay where they are."""
    w = _update_clip_workload(optimizer == "lion")
    run = P.Run(w, optimizer=optimizer, update_clipping=True)
    hp = (B.make_hyper(lambda_rel=20.0, clip_mode=B.ADAGC_MODE_AGC) if optimizer == "adamw" else
          B.make_hyper(lr=1e-4, beta1=0.9, beta2=0.99, lambda_rel=20.0, clip_mode=B.ADAGC_MODE_AGC))
    run.gamma.fill_(5.0)
    run.h_gamma[:] = 5.0
    trajectory(run, hp, 4, "agc-" + optimizer, lockstep=True)
    norms, coefs, flags = run.ctx.get_norms()
    kinds = np.array([s.kind for s in w.specs])
    assert flags[kinds == "bias"].all() and (coefs[kinds == "bias"] == 0.0).all()
    assert not flags[kinds == "norm"].any() and (coefs[kinds == "norm"] == 1.0).all()
    big = np.array([s.kind == "matrix" and s.numel > 1000 for s in w.specs])
    assert flags[big].all() and (coefs[big] > 0.0).all() and (coefs[big] < 1.0).all()
    assert (to_numpy(run.gamma) == 5.0).all()                       # no state
    for i in np.nonzero(kinds == "bias")[0]:
        assert not to_numpy(run.params[i]).any()                    # never moved
    # the scratch must have been reserved at creation
    plain = P.Run(W.Workload(w.specs[:3]), mirror=False)
    with pytest.raises(B.AdagcError) as e:
        plain.gpu_step(plain.w.make_grads(1, DEV), B.make_hyper(clip_mode=B.ADAGC_MODE_AGC), 1)
    assert e.value.code == B.ADAGC_ERR_STATE


@pytest.mark.parametrize("optimizer", ["adamw", "lion"])
def test_clippy_mode_update_clipping_by_weight_max(optimizer):
    """Table 2's Clippy row with l-infinity norms: (lambda_rel max|theta| + lambda_abs) / (lr max|Delta|)."""
    w = _update_clip_workload(optimizer == "lion")
    run = P.Run(w, optimizer=optimizer, update_clipping=True)
    hp = (B.make_hyper(lr=0.05, lambda_rel=0.5, lambda_abs=0.02, clip_mode=B.ADAGC_MODE_CLIPPY) if optimizer == "adamw"
          else B.make_hyper(lr=0.05, beta1=0.9, beta2=0.99, lambda_rel=0.5, lambda_abs=0.02, clip_mode=B.ADAGC_MODE_CLIPPY))
    clipped = trajectory(run, hp, 4, "clippy-" + optimizer, lockstep=True)
    assert 10 < clipped < 4 * w.n_tensors - 10                      # clipped and unclipped tensors both occurred
    # the same context goes back to the paper's method: the update coefficient must not linger
    hp0 = B.make_hyper(t_start=0) if optimizer == "adamw" else B.make_hyper(lr=1e-4, beta1=0.9, beta2=0.99, t_start=0)
    run.gamma.fill_(1e-2)
    for step in (5, 6):
        run.h_params = [to_numpy(t) for t in run.params]
        run.h_m = [to_numpy(t) for t in run.m]
        if run.v is not None:
            run.h_v = [to_numpy(t) for t in run.v]
        run.h_gamma = to_numpy(run.gamma)
        grads = w.make_grads(step, DEV)
        norms, coefs, flags = run.gpu_step(grads, hp0, step)
        rn, rc, rf, thr = run.oracle_step([to_numpy(g) for g in grads], hp0, step)
        P.check_scalars("clippy-then-adagc step %d" % step, norms, coefs, flags, to_numpy(run.gamma), rn, rc, rf,
                        run.h_gamma, thr)
        exempt = None
        if optimizer == "lion":
            continue                                                  # the AdamW run checks the state below
        run.compare_state("clippy-then-adagc step %d" % step, exempt)


def _telemetry_case(optimizer, w, hp, name, **knobs):
    run = P.Run(w, optimizer=optimizer, telemetry=True, **knobs)
    plain = P.Run(w, optimizer=optimizer, mirror=False)
    for step in range(1, 5):
        grads = w.make_grads(step, DEV)
        grads_np = [to_numpy(g) for g in grads]
        run.h_params = [to_numpy(t) for t in run.params]          # lockstep
        run.h_m = [to_numpy(t) for t in run.m]
        if run.v is not None:
            run.h_v = [to_numpy(t) for t in run.v]
        run.h_gamma = to_numpy(run.gamma)
        before = [x.copy() for x in run.h_params]
        run.gpu_step(grads, hp, step)
        plain.gpu_step(grads, hp, step)
        run.oracle_step(grads_np, hp, step)
        m_n, v_n, u_n = run.ctx.get_state_norms()
        for i in range(w.n_tensors):
            rm, rv, ru = oracle.state_norms(before[i], run.h_params[i], run.h_m[i],
                                            run.h_v[i] if run.h_v is not None else None)
            tag = "%s step %d tensor %d" % (name, step, i)
            assert m_n[i] == pytest.approx(rm, rel=P.RTOL, abs=1e-30), tag + " |m|"
            assert v_n[i] == pytest.approx(rv, rel=P.RTOL, abs=1e-30), tag + " |v|"
            # the update is a difference of stored fp32 values: allow one fp32 rounding of theta per element
            slack = 6e-8 * float(np.linalg.norm(run.h_params[i].astype(np.float64)))
            assert abs(u_n[i] - ru) <= P.RTOL * ru + slack, tag + " |update|"
        if optimizer == "lion":
            assert (v_n == 0).all()
    # telemetry does not change the step itself
    for a, b in zip(run.params + run.m + [run.gamma], plain.params + plain.m + [plain.gamma]):
        assert torch.equal(a, b)
    code = None
    try:
        plain.ctx.get_state_norms()
    except B.AdagcError as e:
        code = e.code
    assert code == B.ADAGC_ERR_STATE


def test_telemetry_state_norms_adamw():
    specs = W.llama_like_list(1, 256, 4, 2, 896, 4000) + W.ragged_stress_list(40, 1 << 15, None)
    w = W.config3(specs)
    w.spikes = {3: (np.arange(0, len(specs), 4), 50.0)}
    _telemetry_case("adamw", w, B.make_hyper(), "telemetry-adamw")


def test_telemetry_state_norms_lion_bf16_grads():
    specs = W.llama_like_list(1, 256, 4, 2, 896, 4000)
    w = W.config4(specs)
    w.spikes = {3: (np.arange(0, len(specs), 4), 50.0)}
    _telemetry_case("lion", w, B.make_hyper(lr=1e-4, beta1=0.9, beta2=0.99), "telemetry-lion", update_split=1)


# --------------------------------------------------------------------------- determinism, state, errors

def test_run_to_run_and_permutation_determinism():
    specs = W.ragged_stress_list(300, 1 << 16, None)
    w = W.Workload(specs)
    hp = B.make_hyper()

    def run_once(order):
        ws = W.Workload([specs[i] for i in order])
        ws.sigma = w.sigma[order]
        run = P.Run(ws, mirror=False)
        out = None
        for step in range(1, 4):
            grads = [w.make_grad(i, step, DEV) for i in order]     # same bits per original tensor
            for k, i in enumerate(order):
                if step == 1:
                    run.params[k].copy_(w.init_param(i, DEV))
            out = run.gpu_step(grads, hp, step)
        state = [(to_numpy(run.params[k]), to_numpy(run.m[k]), to_numpy(run.v[k])) for k in range(len(order))]
        return out, to_numpy(run.gamma), state

    ident = np.arange(len(specs))
    a = run_once(ident)
    b = run_once(ident)
    perm = np.random.default_rng(5).permutation(len(specs))
    c = run_once(perm)
    for x, y in zip(a[0], b[0]):
        assert np.array_equal(x, y)
    assert np.array_equal(a[1], b[1])
    for k, i in enumerate(perm):
        assert a[0][0][i] == c[0][0][k] and a[0][1][i] == c[0][1][k] and a[1][i] == c[1][k]
        for x, y in zip(a[2][i], c[2][k]):
            assert np.array_equal(x, y)
    for sa, sb in zip(a[2], b[2]):
        for x, y in zip(sa, sb):
            assert np.array_equal(x, y)


def test_context_holds_no_algorithm_state():
    """Destroying and re-creating the context mid-run changes nothing: all state is the caller's."""
    w = W.config1()
    hp = B.make_hyper()
    a = P.Run(w, mirror=False)
    b = P.Run(w, mirror=False)
    for step in range(1, 7):
        grads = w.make_grads(step, DEV)
        a.gpu_step(grads, hp, step)
        if step == 4:
            b.ctx.close()
            b.ctx = B.AdaGC(w.numels)
        b.gpu_step(grads, hp, step)
    for x, y in zip(a.params + a.m + a.v + [a.gamma], b.params + b.m + b.v + [b.gamma]):
        assert torch.equal(x, y)


def test_step_errors_leave_state_untouched():
    numels = [100, 5000]
    specs = [W.TensorSpec("t%d" % i, (n,), "matrix") for i, n in enumerate(numels)]
    w = W.Workload(specs, bf16_copy=True)
    run = P.Run(w, mirror=False)
    grads = w.make_grads(1, DEV)
    before = [t.clone() for t in run.params + run.m + run.v + [run.gamma]]
    hp = B.make_hyper()
    L = B.lib()

    def code(fn):
        with pytest.raises(B.AdagcError) as e:
            fn()
        return e.value.code

    assert code(lambda: run.ctx.step(run.params, grads, run.m, run.v, run.gamma, hp, 0)) == B.ADAGC_ERR_INVALID_ARG
    assert code(lambda: run.ctx.step(run.params, grads, run.m, None, run.gamma, hp, 1)) == B.ADAGC_ERR_INVALID_ARG
    bad = B.make_hyper(beta1=1.0)
    assert code(lambda: run.ctx.step(run.params, grads, run.m, run.v, run.gamma, bad, 1)) == B.ADAGC_ERR_INVALID_ARG
    bad = B.make_hyper(clip_mode=99)
    assert code(lambda: run.ctx.step(run.params, grads, run.m, run.v, run.gamma, bad, 1)) == B.ADAGC_ERR_INVALID_ARG
    bad = B.make_hyper(lambda_rel=float("nan"))
    assert code(lambda: run.ctx.step(run.params, grads, run.m, run.v, run.gamma, bad, 1)) == B.ADAGC_ERR_INVALID_ARG
    nullp = (ctypes.c_void_p * 2)(run.params[0].data_ptr(), None)
    assert code(lambda: run.ctx.step(nullp, grads, run.m, run.v, run.gamma, hp, 1)) == B.ADAGC_ERR_INVALID_ARG
    # bf16 copies announced but never registered
    ctx2 = B.AdaGC(numels, has_bf16_param_copy=True)
    assert code(lambda: ctx2.step(run.params, grads, run.m, run.v, run.gamma, hp, 1)) == B.ADAGC_ERR_STATE
    ctx2.close()
    ctx3 = B.AdaGC(numels)
    assert code(lambda: ctx3.set_param_copies(run.copies)) == B.ADAGC_ERR_STATE
    ctx3.close()
    assert L.adagc_get_norms(run.ctx._ctx, None, None, None, 3, None) == B.ADAGC_ERR_INVALID_ARG
    torch.cuda.synchronize()
    for x, y in zip(before, run.params + run.m + run.v + [run.gamma]):
        assert torch.equal(x, y)
    # and the context still works afterwards
    run.gpu_step(grads, hp, 1)
    assert not torch.equal(before[0], run.params[0])


def test_launch_tuning_knobs_do_not_change_results():
    """grid size, unroll depth and non-temporal hints are scheduling choices only."""
    specs = W.llama_like_list(1, 256, 4, 2, 896, 4000)
    w = W.config3(specs)
    hp = B.make_hyper()
    outs = []
    for kw in (dict(), dict(grid_blocks=7), dict(unroll=1), dict(unroll=4, nontemporal=1),
               dict(grid_blocks=100000, unroll=2, nontemporal=2), dict(schedule=1), dict(schedule=7, grid_blocks=50),
               dict(schedule=1000000), dict(grid_blocks=1024, schedule=2, unroll=1, nontemporal=2),
               dict(schedule=8), dict(schedule=2, schedule_run=1), dict(schedule=4, schedule_run=3),
               dict(update_split=1), dict(update_split=2, grid_blocks=33), dict(update_split=4, schedule=3),
               dict(update_split=16, unroll=1), dict(update_split=8, unroll=2, nontemporal=2)):
        run = P.Run(w, mirror=False, **kw)
        for step in range(1, 4):
            run.gpu_step(w.make_grads(step, DEV), hp, step)
        outs.append([to_numpy(t) for t in run.params + run.m + run.v + run.copies + [run.gamma]])
    for other in outs[1:]:
        for x, y in zip(outs[0], other):
            assert np.array_equal(x, y)


def test_steps_on_a_side_stream_and_profile_events():
    w = W.config1()
    run = P.Run(w, mirror=False)
    ref = P.Run(w, mirror=False)
    hp = B.make_hyper()
    side = torch.cuda.Stream()
    run.ctx.profile_begin(8)
    grads = [w.make_grads(s, DEV) for s in range(1, 4)]
    torch.cuda.synchronize()
    for step in range(1, 4):
        run.ctx.step(run.params, grads[step - 1], run.m, run.v, run.gamma, hp, step, stream=side.cuda_stream)
        ref.ctx.step(ref.params, grads[step - 1], ref.m, ref.v, ref.gamma, hp, step)
    n1 = run.ctx.get_norms(stream=side.cuda_stream)
    ms = run.ctx.profile_end()
    n2 = ref.ctx.get_norms()
    torch.cuda.synchronize()
    assert ms.shape == (3, 3) and (ms > 0).all() and (ms < 1000).all()
    for x, y in zip(n1, n2):
        assert np.array_equal(x, y)
    for x, y in zip(run.params, ref.params):
        assert torch.equal(x, y)


def test_alternating_pointer_sets_match_a_single_set():
    """A caller that alternates between gradient buffers changes the pointer table on every step: the table is
    re-uploaded through the ring of staging tables, with the host running ahead of the GPU.  Twelve steps issued
    back to back over three rotating gradient sets must give exactly what the same gradients give from one buffer."""
    specs = W.gpt2_like_list(2, 128, 512, 1024, 0)
    w = W.Workload(specs, spikes=W.forced_spike_schedule(len(specs), 12, {5, 9}, 4, 60.0))
    hp = B.make_hyper()
    a = P.Run(w, mirror=False)
    b = P.Run(w, mirror=False)
    sets = [w.make_grads(1, DEV) for _ in range(3)]
    single = w.make_grads(1, DEV)
    all_grads = [w.make_grads(step, DEV) for step in range(1, 13)]
    # run a: every step's gradients are copied into the next buffer set of the rotation, steps issued without waiting
    for step in range(1, 13):
        dst = sets[step % 3]
        for d, g in zip(dst, all_grads[step - 1]):
            d.copy_(g)
        a.ctx.step(a.params, dst, a.m, a.v, a.gamma, hp, step)
    # run b: one buffer set
    for step in range(1, 13):
        for d, g in zip(single, all_grads[step - 1]):
            d.copy_(g)
        b.ctx.step(b.params, single, b.m, b.v, b.gamma, hp, step)
    torch.cuda.synchronize()
    for x, y in zip(a.params + a.m + a.v + [a.gamma], b.params + b.m + b.v + [b.gamma]):
        assert torch.equal(x, y)
    assert a.ctx.get_norms()[2].sum() == b.ctx.get_norms()[2].sum()


def test_non_finite_gradient_propagates_like_plain_adamw():
    """A NaN in one tensor's gradient makes that tensor's norm NaN: the comparison with the threshold
    is false, the tensor is not clipped, and the NaN flows into its own state only."""
    numels = [300, 5000, 70]
    rng = np.random.default_rng(3)
    grads = [rng.standard_normal(n).astype(np.float32) * 0.01 for n in numels]
    grads[1][1234] = np.nan
    grads[2][5] = np.inf
    hp = B.make_hyper(t_start=0)
    run, got, ref = _single(numels, grads, [1.0, 1.0, 1.0], hp, 2)
    norms, coefs, flags = got
    assert np.isnan(norms[1]) and coefs[1] == 1.0 and flags[1] == 0
    assert np.isinf(norms[2]) and flags[2] == 1 and coefs[2] == 0.0            # thr / inf = 0
    assert np.isnan(ref[0][1]) and ref[1][1] == 1.0 and ref[2][1] == 0 and ref[2][2] == 1
    assert np.isnan(to_numpy(run.gamma)[1]) and np.isnan(run.h_gamma[1])
    P.assert_close("finite tensor theta", to_numpy(run.params[0]), run.h_params[0])
    P.assert_close("finite tensor m", to_numpy(run.m[0]), run.h_m[0])
    gpu_m1, ref_m1 = to_numpy(run.m[1]), run.h_m[1]
    assert np.array_equal(np.isnan(gpu_m1), np.isnan(ref_m1)) and int(np.isnan(gpu_m1).sum()) == 1
    # inf * 0 = NaN in the clipped gradient of the inf element, on both sides
    assert np.array_equal(np.isnan(to_numpy(run.m[2])), np.isnan(run.h_m[2]))


def test_remaining_dtype_combinations():
    """AdamW with bf16 gradients (no copy) and Lion with fp32 gradients plus the bf16 copy."""
    specs = W.llama_like_list(1, 256, 4, 2, 896, 4000)
    w = W.Workload(specs, grad_dtype=torch.bfloat16, spikes={3: (np.arange(0, len(specs), 3), 40.0)})
    trajectory(P.Run(w), B.make_hyper(), 4, "adamw-bf16-grads", lockstep=True)
    w = W.Workload(specs, bf16_copy=True, spikes={3: (np.arange(0, len(specs), 3), 40.0)})
    trajectory(P.Run(w, optimizer="lion"), B.make_hyper(lr=1e-4, beta1=0.9, beta2=0.99), 4, "lion-fp32-grads-copy",
               lockstep=True)


def test_list_of_one_tensor_of_one_element():
    hp = B.make_hyper(t_start=0)
    run, got, ref = _single([1], [np.array([0.5])], [0.25], hp, 9)
    norms, coefs, flags = got
    assert norms[0] == 0.5 and flags[0] == 1 and coefs[0] == np.float32(np.float32(1.04) * 0.25 / 0.5)
    P.check_scalars("one-element", norms, coefs, flags, to_numpy(run.gamma), ref[0], ref[1], ref[2], run.h_gamma, ref[3])
    run.compare_state("one-element")


# --------------------------------------------------------------------------- the published schedule, and a seeded sweep

@pytest.mark.parametrize("quiet_warmup", [False, True])
def test_paper_default_schedule_warmup_100_then_adagc(quiet_warmup):
    """Alg. 1 with the defaults of Sec. 4.2 / 5.2 (lambda_rel 1.04, beta 0.99, T_start 100, lambda_abs 1.0) run
    free for 150 steps on the tiny transformer list: 100 GlobalGC warm-up steps with the running minimum, then
    per-tensor AdaGC with spikes.  The oracle is never re-seeded from the device.
    quiet_warmup=False: the model's norm is far above lambda_abs and one warm-up step spikes, so every step of the
    warm-up clips globally and the thresholds start low (every tensor clips afterwards).
    quiet_warmup=True: gradients are scaled so that the model's norm stays below lambda_abs; the thresholds start
    at each tensor's smallest norm and only some tensors clip afterwards."""
    specs = W.tiny_transformer_list()
    spike_steps = {101, 120, 135} if quiet_warmup else {50, 101, 120, 135}
    w = W.Workload(specs, spikes=W.forced_spike_schedule(len(specs), 150, spike_steps, 3, 100.0))
    if quiet_warmup:
        w.sigma = w.sigma * (0.9 / math.sqrt(sum(float(s) ** 2 * k for s, k in zip(w.sigma, w.numels))))
    hp = B.make_hyper(t_start=100, lambda_abs=1.0)
    run = P.Run(w)
    name = "paper-defaults%s" % (" (quiet warm-up)" if quiet_warmup else "")
    warm_clips, after = 0, []
    for step in range(1, 151):
        grads = w.make_grads(step, DEV)
        norms, coefs, flags = run.gpu_step(grads, hp, step)
        ref_norms, ref_coefs, ref_flags, thr = run.oracle_step([to_numpy(g) for g in grads], hp, step)
        P.check_scalars("%s step %d" % (name, step), norms, coefs, flags, to_numpy(run.gamma), ref_norms,
                        ref_coefs, ref_flags, run.h_gamma, None if step <= 100 else thr)
        if step <= 100:
            assert np.all(coefs == coefs[0]) and np.all(flags == flags[0])   # one decision for the whole model
            warm_clips += int(flags[0])
        else:
            after.append(int(flags.sum()))
        if step in (50, 100, 101, 120, 150):
            differ = run.compare_state("%s step %d" % (name, step))
            say("%s step %d: %d values not bit-identical, %d clipped" % (name, step, differ, int(flags.sum())))
    if quiet_warmup:
        assert warm_clips == 0 and 0 < min(after) < len(specs) and max(after) > min(after)
    else:
        assert warm_clips == 100 and min(after) == len(specs)


def test_seeded_sweep_of_lists_modes_and_dtypes():
    """32 seeded random cases: list length, sizes next to every vector / chunk boundary, optimizer, gradient
    type, bf16 copy, clipping mode, warm-up length, thresholds and launch knobs, three lockstep steps each."""
    c = B.adagc_chunk_elems()
    pool = [1, 2, 3, 4, 5, 7, 8, 9, 63, 64, 65, 255, 256, 257, 1020, 1023, 1024, 1025, 1027, 4095, 4097,
            c - 4, c - 1, c, c + 1, c + 4, 2 * c - 1, 2 * c + 2, 3 * c + 3, 50001]
    rng = np.random.default_rng(20250211)
    for case in range(32):
        n = int(rng.integers(1, 13))
        numels = [int(pool[k]) for k in rng.integers(0, len(pool), n)]
        lion = bool(rng.integers(0, 2))
        bf16g = bool(rng.integers(0, 2))
        copy = bool(rng.integers(0, 2))
        mode = int(rng.integers(0, 3))
        t_start = int(rng.integers(0, 4))
        knobs = dict(unroll=int(rng.choice([0, 1, 2, 4])), schedule=int(rng.choice([0, 1, 3, 8])),
                     grid_blocks=int(rng.choice([0, 0, 5, 64])), nontemporal=int(rng.choice([0, 1, 2])),
                     update_split=int(rng.choice([0, 1, 2, 4])), schedule_run=int(rng.choice([0, 1, 3])))
        specs = [W.TensorSpec("t%d" % i, (k,), "matrix") for i, k in enumerate(numels)]
        spikes = {2: (np.arange(0, n, 2), 30.0), 3: (np.arange(1, n, 2), 30.0)}
        w = W.Workload(specs, seed=1000 + case, spikes=spikes, bf16_copy=copy,
                       grad_dtype=torch.bfloat16 if bf16g else torch.float32)
        # a GlobalGC threshold near the unspiked model norm, so that some steps clip and some do not
        model_norm = math.sqrt(sum(float(s) ** 2 * k for s, k in zip(w.sigma, numels)))
        hp = B.make_hyper(lr=1e-4 if lion else 3e-4, beta2=0.99 if lion else 0.95, t_start=t_start,
                          clip_mode=mode, lambda_abs=float(rng.choice([0.5, 2.0, math.inf])) * model_norm,
                          lambda_rel=float(rng.choice([1.04, 1.0, 2.0])))
        name = "sweep case %d (%s, %s grads%s, mode %d, t_start %d, %d tensors, %s)" % (
            case, "lion" if lion else "adamw", "bf16" if bf16g else "fp32", ", copy" if copy else "", mode, t_start,
            n, knobs)
        say(name)
        run = P.Run(w, optimizer="lion" if lion else "adamw", **knobs)
        if t_start == 0:       # no initialising step: the caller provides gamma
            g0 = np.array([0.7 * float(s) * math.sqrt(k) for s, k in zip(w.sigma, numels)], dtype=np.float32)
            if mode == B.ADAGC_MODE_GLOBAL_ADAGC:
                g0[0] = np.float32(0.7 * model_norm)
            run.gamma.copy_(torch.from_numpy(g0))
        trajectory(run, hp, 3, name, lockstep=True)
        run.ctx.close()


# --------------------------------------------------------------------------- the comparisons have teeth

class _ZeroHead(W.Workload):
    """Gradients whose first three elements are exactly zero (Lion's sign(0) case while m is still zero)."""

    def fill_grad(self, out, i, step):
        super().fill_grad(out, i, step)
        out[:3] = 0
        return out


def _teeth_scenarios():
    """Two short lockstep runs that between them exercise every statement of Alg. 1 and of the Lion rule:
    warm-up with an active global clip and the running minimum, AdaGC with clipped and unclipped tensors,
    AdamW with a bf16 copy, Lion on bf16 gradients with exact zeros."""
    specs = W.llama_like_list(1, 64, 4, 2, 224, 500)
    spikes = {4: (np.arange(0, len(specs), 2), 40.0), 5: (np.arange(1, len(specs), 2), 40.0)}
    w = W.Workload(specs, spikes=spikes, bf16_copy=True)
    model_norm = math.sqrt(sum(float(s) ** 2 * k for s, k in zip(w.sigma, w.numels)))
    trajectory(P.Run(w), B.make_hyper(t_start=2, lambda_abs=0.5 * model_norm, eps=1e-3), 6, "teeth-adamw", lockstep=True)
    w = _ZeroHead(specs, spikes=spikes, grad_dtype=torch.bfloat16)
    trajectory(P.Run(w, optimizer="lion"), B.make_hyper(lr=1e-4, beta1=0.9, beta2=0.99), 5, "teeth-lion", lockstep=True)
    # ZClip: two gathering steps (the first globally clipped), then clipped and unclipped z-score steps
    every = np.arange(len(specs))
    scale = {1: 1.5, 2: 1.0, 3: 0.9, 4: 3.0, 5: 1.0, 6: 0.8, 7: 1.1}
    w = W.Workload(specs, spikes={t: (every, f) for t, f in scale.items()})
    hp = B.make_hyper(t_start=2, lambda_abs=1.2 * model_norm, clip_mode=B.ADAGC_MODE_ZCLIP, ema_beta=0.75, z_thres=2.0)
    trajectory(P.Run(w), hp, 7, "teeth-zclip", lockstep=True)
    # AGC and Clippy: clipped and unclipped tensors, with weight decay, AdamW and Lion
    w = W.Workload(W.gpt2_like_list(1, 64, 256, 300, 0), sigma_lo=1e-3, sigma_hi=1e-1)
    trajectory(P.Run(w, update_clipping=True), B.make_hyper(lambda_rel=20.0, clip_mode=B.ADAGC_MODE_AGC, eps=1e-3), 3,
               "teeth-agc", lockstep=True)
    trajectory(P.Run(w, update_clipping=True), B.make_hyper(lr=0.05, lambda_rel=0.5, lambda_abs=0.02,
                                                            clip_mode=B.ADAGC_MODE_CLIPPY), 3, "teeth-clippy", lockstep=True)
    trajectory(P.Run(w, optimizer="lion", update_clipping=True),
               B.make_hyper(lr=1e-3, beta1=0.9, beta2=0.99, lambda_rel=20.0, clip_mode=B.ADAGC_MODE_AGC), 3, "teeth-agc-lion",
               lockstep=True)


def test_parity_comparisons_notice_a_wrong_oracle(tmp_path):
    """Plant each mistake of tests/planted.py in a copy of the CPU oracle (the GPU library is untouched) and run
    the scenarios: the comparison must fail for every mistake that changes what a step computes.  Two entries
    are left to the CPU pins: ties of the bf16 rounding (the copy is compared to within one bf16 ulp) and
    '>=' for '>' in Eq. 3 and in ZClip (differs only at exact equality)."""
    import planted
    _teeth_scenarios()                                  # the real oracle agrees
    cpu_only = {"bf16 ties always round up", "clip on >= instead of >", "ZClip: clip on >= instead of >"}
    unnoticed = []
    for k, (what, _, _) in enumerate(planted.MISTAKES):
        if what in cpu_only:
            continue
        with planted.wrong_oracle(tmp_path, k):
            try:
                _teeth_scenarios()
                unnoticed.append(what)
            except AssertionError:
                pass
        say("planted: %s -> %s" % (what, "NOT NOTICED" if unnoticed and unnoticed[-1] == what else "noticed"))
    assert not unnoticed, "mistakes the GPU parity comparison does not notice: %s" % unnoticed
