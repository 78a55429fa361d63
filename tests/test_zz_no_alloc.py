"""adagc_step_static (the step for callers that cannot allocate) against adagc_step, through the C ABI.
Both run the same kernels, so every output must be bit-identical: theta, m, v, bf16 copies, gamma,
norms, coefficients, clip flags.  Two calls in a row share the library's fixed device array, the second
on a smaller list than the first."""
import numpy as np
import pytest
import torch

from paper_2502_11034_amd import binding as B
from paper_2502_11034_amd import workloads as W
from paper_2502_11034_amd.workloads import to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _state(w, optimizer, seed):
    params, m, v, copies = w.make_state(DEV, optimizer)
    gen = torch.Generator(device=DEV).manual_seed(seed)
    for t in m:
        t.normal_(0, 1e-3, generator=gen)
    if v is not None:
        for t in v:
            t.normal_(0, 1e-3, generator=gen).square_()
    return params, m, v, copies


def _clone(lst):
    return None if lst is None else [t.clone() for t in lst]


def _same(name, a, b):
    for i, (x, y) in enumerate(zip(a, b)):
        assert np.array_equal(to_numpy(x).view(np.uint8), to_numpy(y).view(np.uint8)), "%s: tensor %d differs" % (name, i)


def _both(w, optimizer, hp, step, gamma0, name):
    """One step through adagc_step and one through adagc_step_static from the same state; compare all outputs."""
    lion = optimizer == "lion"
    opt = B.ADAGC_OPT_LION if lion else B.ADAGC_OPT_ADAMW
    gd = B.ADAGC_GRAD_BF16 if w.grad_dtype == torch.bfloat16 else B.ADAGC_GRAD_F32
    params, m, v, copies = _state(w, optimizer, 5)
    grads = w.make_grads(step, DEV)
    a = (params, m, v, copies, gamma0.clone())
    b = (_clone(params), _clone(m), _clone(v), _clone(copies), gamma0.clone())

    ctx = B.AdaGC(w.numels, opt, gd, w.bf16_copy)
    if copies is not None:
        ctx.set_param_copies(a[3])
    ctx.step(a[0], grads, a[1], a[2], a[4], hp, step)
    norms, coefs, flags = ctx.get_norms()
    ctx.close()

    n = w.n_tensors
    o_norm = torch.full((n,), -1.0, dtype=torch.float32, device=DEV)
    o_coef = torch.full((n,), -1.0, dtype=torch.float32, device=DEV)
    o_flag = torch.full((n,), 7, dtype=torch.uint8, device=DEV)
    B.adagc_step_static(w.numels, b[0], grads, b[1], b[2], b[4], hp, step, optimizer=opt, grad_dtype=gd,
                        params_bf16=b[3], out_norms=o_norm, out_coefs=o_coef, out_clipped=o_flag)
    torch.cuda.synchronize()

    assert np.array_equal(to_numpy(o_norm).view(np.uint32), norms.view(np.uint32)), name + " norms"
    assert np.array_equal(to_numpy(o_coef).view(np.uint32), coefs.view(np.uint32)), name + " coefs"
    assert np.array_equal(to_numpy(o_flag), flags), name + " flags"
    assert np.array_equal(to_numpy(a[4]).view(np.uint32), to_numpy(b[4]).view(np.uint32)), name + " gamma"
    _same(name + " theta", a[0], b[0])
    _same(name + " m", a[1], b[1])
    if v is not None:
        _same(name + " v", a[2], b[2])
    if copies is not None:
        _same(name + " bf16 copies", a[3], b[3])
    print("%s: %d tensors, %d params, %d clipped: bit-identical to adagc_step" % (name, n, w.total_params, int(flags.sum())),
          flush=True)
    return int(flags.sum())


def test_static_step_matches_adagc_step_on_two_calls_in_a_row():
    # first call: 301 ragged tensors (several argument batches), sizes 1 .. 2^18, plus one of 5 chunks + a tail
    big = W.Workload(W.ragged_stress_list(300, 1 << 18, (5 * 16384 + 77,)), bf16_copy=True)
    gamma = torch.tensor(big.sigma * np.sqrt(np.array(big.numels)), dtype=torch.float32, device=DEV)
    gamma[::3] *= 0.5                                # a third of the tensors clip
    clipped = _both(big, "adamw", B.make_hyper(t_start=0), 4, gamma, "static step, first call (AdamW, bf16 copy)")
    assert 50 < clipped < 300
    # second call, smaller list, other optimizer and gradient type: stale rows of the first call lie behind it
    small = W.config4(W.llama_like_list(1, 256, 4, 2, 512, 1000))
    gamma = torch.tensor(small.sigma * np.sqrt(np.array(small.numels)), dtype=torch.float32, device=DEV)
    gamma[::2] *= 0.5
    clipped = _both(small, "lion", B.make_hyper(lr=1e-4, beta2=0.99, t_start=0), 9, gamma,
                    "static step, second call (Lion, bf16 grads)")
    assert clipped >= 3
    # third: the warm-up branch (one coefficient for the model) on the small list
    hp = B.make_hyper(t_start=10, lambda_abs=0.01)
    clipped = _both(small, "lion", hp, 3, gamma, "static step, warm-up branch")
    assert clipped == small.n_tensors


def test_static_step_rejects_what_does_not_fit():
    hp = B.make_hyper()
    one = torch.zeros(16, device=DEV)
    g1 = torch.zeros(1, device=DEV)
    # too many chunks: one tensor of (max chunks + 1) chunks; rejected before any pointer is used
    n = (B.ADAGC_STATIC_MAX_CHUNKS + 1) * B.adagc_chunk_elems()
    with pytest.raises(B.AdagcError) as e:
        B.adagc_step_static([n], [one], [one], [one], [one], g1, hp, 1)
    assert e.value.code == B.ADAGC_ERR_TOO_LARGE
    # too many tensors
    k = B.ADAGC_STATIC_MAX_TENSORS + 1
    with pytest.raises(B.AdagcError) as e:
        B.adagc_step_static([1] * k, [one] * k, [one] * k, [one] * k, [one] * k, g1, hp, 1)
    assert e.value.code == B.ADAGC_ERR_TOO_LARGE
    # launch tuning is not available here
    L = B.lib()
    import ctypes
    cfg = B.adagc_config(0, 0, 0, 1, 0, 0, 0, 0, 0, 0, 0)     # telemetry = 1
    descs = B._descs([16])
    p = B.ptr_array([one])
    rc = L.adagc_step_static(ctypes.cast(descs, ctypes.c_void_p), 1, ctypes.byref(cfg), p, p, p, p, None,
                             g1.data_ptr(), ctypes.byref(hp), 1, None, None, None, None)
    assert rc == B.ADAGC_ERR_INVALID_ARG
