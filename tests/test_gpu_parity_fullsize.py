"""Full-size GPU parity, in the launch configuration the benchmark times: the whole
Llama-3-8B-shaped list (AdamW + bf16 copy; Lion + bf16 gradients) and the 20 001-tensor ragged
list, resident on one GPU.  The oracle cannot replay 8e9 parameters in seconds, so:
  - per-tensor scalars (norm, coefficient, clip flag, gamma) are checked for EVERY tensor on the
    spike step, from a streamed download of the gradients;
  - the elementwise update is checked in lockstep (oracle starts from the device's pre-step
    state) on a subset that contains the largest tensor, the smallest, tensors of every shape
    class, and spiked tensors.
Tensors are independent under the per-tensor rule, so a subset loses nothing but coverage."""
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


def f32(x):
    return float(np.float32(x))


def run_fullsize(w, optimizer, hp, steps, subset, scalar_step, name, early_subset=None):
    """early_subset: the (smaller) subset checked on the steps before scalar_step; the full subset,
    which holds the largest tensor, is replayed by the oracle on scalar_step only (time)."""
    lion = optimizer == "lion"
    run = P.Run(w, optimizer=optimizer, mirror=False)
    ohp = P.oracle_hyper(hp, run.optimizer, run.grad_dtype)
    say("%s: %d tensors, %d params resident" % (name, w.n_tensors, w.total_params))
    full_subset = subset
    for step in range(1, steps + 1):
        subset = full_subset if (step == scalar_step or early_subset is None) else early_subset
        pre = {}
        for i in subset:
            pre[i] = (to_numpy(run.params[i]), to_numpy(run.m[i]),
                      to_numpy(run.v[i]) if run.v is not None else None)
        gamma_prev = to_numpy(run.gamma)
        grads = w.make_grads(step, DEV)
        norms, coefs, flags = run.gpu_step(grads, hp, step)
        gamma_new = to_numpy(run.gamma)
        warm = (step - 1) < hp.t_start

        if step == scalar_step:
            lam, beta = f32(hp.lambda_rel), f32(hp.ema_beta)
            rn = np.zeros(w.n_tensors)
            rc = np.zeros(w.n_tensors)
            rf = np.zeros(w.n_tensors, np.uint8)
            rg = np.zeros(w.n_tensors, np.float32)
            for i in range(w.n_tensors):
                rn[i] = oracle.l2_norm(to_numpy(grads[i]))
                h, g_new, c = oracle.adagc_rule(rn[i], float(gamma_prev[i]), lam, beta)
                rc[i], rf[i], rg[i] = h, c, np.float32(g_new)
            thr = lam * gamma_prev.astype(np.float64)
            P.check_scalars("%s step %d all tensors" % (name, step), norms, coefs, flags, gamma_new,
                            rn, rc, rf, rg, thr)
            say("%s step %d: scalars of all %d tensors ok, %d clipped" % (name, step, w.n_tensors, int(rf.sum())))
            if step in w.spikes:
                assert rf[w.spikes[step][0]].all(), "spiked tensors must clip"

        strict = 0
        for i in subset:
            th, mm, vv = pre[i]
            g_np = to_numpy(grads[i])
            gam = gamma_prev[i:i + 1].copy()
            copy = np.zeros(th.size, np.uint16) if run.copies is not None else None
            m_before = mm.copy()
            rn1, rc1, rf1 = oracle.adagc_step([th], [g_np], [mm], [vv] if vv is not None else None, gam, ohp,
                                              step, [copy] if copy is not None else None)
            tag = "%s step %d tensor %d (%s)" % (name, step, i, w.specs[i].name)
            np.testing.assert_allclose(norms[i], rn1[0], rtol=P.RTOL, err_msg=tag)
            np.testing.assert_allclose(coefs[i], rc1[0], rtol=P.RTOL, err_msg=tag)
            np.testing.assert_allclose(gamma_new[i], gam[0], rtol=P.RTOL, err_msg=tag)
            if warm or abs(rn1[0] / (f32(hp.lambda_rel) * float(gamma_prev[i])) - 1.0) > P.BAND:
                assert flags[i] == rf1[0], tag
            ex = run.lion_exempt(i, g_np, m_before, rc1[0], hp) if lion else None
            gpu_theta = to_numpy(run.params[i])
            strict += P.assert_close(tag + " theta", gpu_theta, th, exempt=ex)
            strict += P.assert_close(tag + " m", to_numpy(run.m[i]), mm)
            if vv is not None:
                strict += P.assert_close(tag + " v", to_numpy(run.v[i]), vv)
            if copy is not None:
                P.assert_bf16_copy(tag, to_numpy(run.copies[i]), gpu_theta, th, ex)
            del th, mm, vv, g_np, copy
        say("%s step %d: update within relative 1e-5 on every element of %d tensors (%d values not bit-identical)"
            % (name, step, len(subset), strict))
        del grads, pre
    run.ctx.close()
    del run
    torch.cuda.empty_cache()


def llama_subsets(w, spike_step):
    names = {s.name: i for i, s in enumerate(w.specs)}
    early = [names["l0.attn_norm"], names["l0.k"], names["final_norm"]]
    subset = early + [names["embed"], names["l7.q"], names["l31.down"]]
    spiked = [int(i) for i in w.spikes[spike_step][0]]
    small_spiked = sorted(spiked, key=lambda i: w.numels[i])[:2]
    return sorted(set(subset + small_spiked)), sorted(set(early + small_spiked))


def test_config3_full_size_llama3_8b_adamw():
    w = W.config3()
    assert w.n_tensors == 291 and w.total_params == 8030261248
    full, early = llama_subsets(w, 3)
    run_fullsize(w, "adamw", B.make_hyper(), 3, full, 3, "config3-full", early)


def test_config4_full_size_llama3_8b_lion_bf16_grads():
    w = W.config4()
    hp = B.make_hyper(lr=1e-4, beta1=0.9, beta2=0.99, weight_decay=0.1)
    full, early = llama_subsets(w, 3)
    run_fullsize(w, "lion", hp, 3, full, 3, "config4-full", early)


def test_config5_full_size_ragged_stress():
    w = W.config5()
    assert w.n_tensors == 20001
    sizes = np.array(w.numels)
    rng = np.random.default_rng(7)
    order = np.argsort(sizes)
    subset = sorted(set([int(order[0]), int(order[1]), int(order[-2])] +          # smallest two, largest ragged
                        [int(i) for i in rng.choice(20000, 150, replace=False)] +
                        [20000]))                                                  # the 128256x4096 tensor
    early = [i for i in subset if w.numels[i] <= (1 << 20)]
    run_fullsize(w, "adamw", B.make_hyper(), 2, subset, 2, "config5-full", early)


def test_one_tensor_beyond_2_to_31_elements():
    """Maximum sizes: a single tensor of 2^31 + 12345 elements (8.6 GB per fp32 array), so that element
    offsets pass 2^31 and byte offsets pass 2^33.  The oracle computes the full norm; the update is
    replayed on slices at the start, across the 2^31-element mark and at the ragged end."""
    n = (1 << 31) + 12345
    dev = DEV
    gen = torch.Generator(device=dev).manual_seed(77)
    g = torch.empty(n, dtype=torch.float32, device=dev).normal_(0, 3e-3, generator=gen)
    p = torch.empty(n, dtype=torch.float32, device=dev).normal_(0, 0.02, generator=gen)
    m = torch.empty(n, dtype=torch.float32, device=dev).normal_(0, 1e-3, generator=gen)
    v = torch.empty(n, dtype=torch.float32, device=dev).normal_(0, 1e-3, generator=gen).square_()
    copy = torch.empty(n, dtype=torch.bfloat16, device=dev)
    gamma = torch.tensor([1.0], dtype=torch.float32, device=dev)
    slices = [(0, 1 << 20), ((1 << 31) - (1 << 19), (1 << 31) + 4096), (n - 70001, n)]
    pre = [(to_numpy(p[a:b]), to_numpy(m[a:b]), to_numpy(v[a:b]), to_numpy(g[a:b])) for a, b in slices]
    hp = B.make_hyper(t_start=0)
    ctx = B.AdaGC([n], has_bf16_param_copy=True)
    assert ctx.num_chunks() == -(-n // B.adagc_chunk_elems())
    ctx.set_param_copies([copy])
    ctx.step([p], [g], [m], [v], gamma, hp, 3)
    norms, coefs, flags = ctx.get_norms()
    ref_norm = oracle.l2_norm(to_numpy(g))
    h, gamma_new, clipped = oracle.adagc_rule(ref_norm, 1.0, f32(hp.lambda_rel), f32(hp.ema_beta))
    say("2^31+ tensor: norm %.6f (ref %.6f), h %.6f, clipped %d" % (norms[0], ref_norm, coefs[0], clipped))
    assert clipped and flags[0] == 1
    np.testing.assert_allclose(norms[0], ref_norm, rtol=P.RTOL)
    np.testing.assert_allclose(coefs[0], h, rtol=P.RTOL)
    np.testing.assert_allclose(to_numpy(gamma)[0], np.float32(gamma_new), rtol=P.RTOL)
    ohp = P.oracle_hyper(hp, 0, 0)
    for (a, b), (th, mm, vv, gg) in zip(slices, pre):
        ref_copy = np.zeros(b - a, np.uint16)
        oracle.adamw_update(th, mm, vv, gg, h, ohp, 3, ref_copy)
        tag = "2^31+ tensor slice [%d, %d)" % (a, b)
        gpu_theta = to_numpy(p[a:b])
        P.assert_close(tag + " theta", gpu_theta, th)
        P.assert_close(tag + " m", to_numpy(m[a:b]), mm)
        P.assert_close(tag + " v", to_numpy(v[a:b]), vv)
        P.assert_bf16_copy(tag, to_numpy(copy[a:b]), gpu_theta, th)
    ctx.close()
