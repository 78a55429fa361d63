"""Helpers of the GPU parity tests: run the HIP path and the CPU oracle on the same seeded
inputs and compare element by element.

Tolerances:
  - segment table, tensor indexing: bit-exact.
  - clip / no-clip decision: bit-exact for every tensor whose norm is not within 1e-6 relative
    of its threshold (inside that band either outcome is accepted: h is continuous there).
  - fp32 norms, coefficients, gamma: relative 1e-5.
  - updated theta / m / v: strict relative 1e-5 on every element, |gpu - ref| <= 1e-5*|ref|.
    Both sides evaluate the update in double and round each stored value once, so in practice the
    arrays are bit-identical except for a handful of 1-ulp differences where the double results
    straddle an fp32 rounding boundary; the number of elements that are not bit-identical is
    returned and printed.
  - bf16 copies: exactly RNE(gpu theta), and at most 1 bf16 ulp from RNE(reference theta).
  - Lion: an element whose interpolation c is within 1e-6 relative of zero may take either sign
    (both sides decide the sign in double with the same operation sequence; never observed).
"""
import numpy as np
import torch

import oracle
from paper_2502_11034_amd import binding as B
from paper_2502_11034_amd.workloads import to_numpy

RTOL = 1e-5
BAND = 1e-6


def oracle_hyper(hp, optimizer, grad_dtype):
    return oracle.Hyper(lr=hp.lr, beta1=hp.beta1, beta2=hp.beta2, eps=hp.eps, weight_decay=hp.weight_decay,
                        lambda_rel=hp.lambda_rel, ema_beta=hp.ema_beta, lambda_abs=hp.lambda_abs,
                        t_start=hp.t_start, optimizer=optimizer, grad_dtype=grad_dtype, clip_mode=hp.clip_mode,
                        z_thres=hp.z_thres)


def rms(x):
    x = x.astype(np.float64)
    return float(np.sqrt(np.mean(x * x))) if x.size else 0.0


def widen_grad(g):
    return (g.astype(np.uint32) << 16).view(np.float32) if g.dtype == np.uint16 else g


def assert_close(name, gpu, ref, rtol=RTOL, exempt=None):
    """Strict per-element relative comparison.  Returns the number of elements that differ at all."""
    gpu64 = gpu.astype(np.float64)
    ref64 = ref.astype(np.float64)
    err = np.abs(gpu64 - ref64)
    bad = ~(err <= rtol * np.abs(ref64))            # also catches NaN on one side only
    bad &= ~(np.isnan(gpu64) & np.isnan(ref64))
    if exempt is not None:
        bad &= ~exempt
    if bad.any():
        k = int(np.argmax(bad))
        raise AssertionError("%s: %d of %d elements beyond relative %g; first at %d: gpu=%r ref=%r"
                             % (name, int(bad.sum()), bad.size, rtol, k, gpu[k], ref[k]))
    return int((gpu.view(np.uint32) != ref.view(np.uint32)).sum())


def assert_close_streamed(name, gpu, ref, exempt_fn=None, envelope_fn=None):
    """assert_close for arrays of 1e8..1e9 elements: a bit comparison first, the relative test only on
    the values that are not bit-identical (the two tests are equivalent: identical bits pass any
    tolerance).  exempt_fn(indices) -> bool array, evaluated only for those values.
    envelope_fn(indices) -> (a, b): the oracle's results at those elements for the two ends of the
    interval in which the tensor's coefficient is defined (see coefficient_interval); a value that
    misses the relative test against the reference passes if it lies between them (within the same
    relative tolerance).  Returns the number of values that are not bit-identical."""
    diff = gpu.view(np.uint32) != ref.view(np.uint32)
    k = int(np.count_nonzero(diff))
    if k == 0:
        return 0
    idx = np.nonzero(diff)[0]
    del diff
    g = gpu[idx].astype(np.float64)
    r = ref[idx].astype(np.float64)
    bad = ~(np.abs(g - r) <= RTOL * np.abs(r))
    bad &= ~(np.isnan(g) & np.isnan(r))
    if exempt_fn is not None and bad.any():
        bad &= ~exempt_fn(idx)
    if envelope_fn is not None and bad.any():
        a, b = envelope_fn(idx[bad])
        lo, hi = np.minimum(a, b).astype(np.float64), np.maximum(a, b).astype(np.float64)
        inside = (g[bad] >= lo - RTOL * np.abs(lo)) & (g[bad] <= hi + RTOL * np.abs(hi))
        bad[np.nonzero(bad)[0]] = ~inside
    if bad.any():
        j = int(np.argmax(bad))
        raise AssertionError("%s: %d of %d elements beyond relative %g; first at %d: gpu=%r ref=%r"
                             % (name, int(bad.sum()), gpu.size, RTOL, int(idx[j]), gpu[idx[j]], ref[idx[j]]))
    return k


def coefficient_interval(h, numel):
    """The interval in which a clipped tensor's coefficient h = lambda*gamma/||g|| is defined.  The paper
    fixes the norm as the l2 norm and no order of summation; two correctly rounded double sums of the same
    N non-negative terms in different orders differ by at most 2(N-1)*2^-53 relative (each is within
    (N-1)*2^-53 of the exact sum), the square root halves that, so h is defined up to N*2^-53 relative.
    An unclipped tensor has h = 1 exactly on both sides: no interval."""
    if h == 1.0:
        return h, h
    d = float(numel) * 2.0 ** -53
    return h * (1.0 - d), h * (1.0 + d)


def bf16_ordered(bits):
    """Map bf16 bit patterns to integers that increase with the represented value."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def assert_bf16_copy(name, gpu_bits, gpu_theta, ref_theta, exempt=None):
    exact = torch.from_numpy(gpu_theta).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(gpu_bits, exact), name + ": bf16 copy is not RNE of the stored fp32 value"
    ref = torch.from_numpy(ref_theta).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    d = np.abs(bf16_ordered(gpu_bits) - bf16_ordered(ref))
    if exempt is not None:
        d = np.where(exempt, 0, d)
    assert int(d.max(initial=0)) <= 1, name + ": bf16 copy more than 1 ulp from the reference"


def check_scalars(name, gpu_norms, gpu_coefs, gpu_flags, gpu_gamma, ref_norms, ref_coefs, ref_flags,
                  ref_gamma, thresholds=None):
    np.testing.assert_allclose(gpu_norms, ref_norms, rtol=RTOL, atol=0, err_msg=name + " norms")
    np.testing.assert_allclose(gpu_coefs, ref_coefs, rtol=RTOL, atol=0, err_msg=name + " coefs")
    np.testing.assert_allclose(gpu_gamma, ref_gamma, rtol=RTOL, atol=0, err_msg=name + " gamma")
    if thresholds is not None:
        with np.errstate(divide="ignore", invalid="ignore"):
            outside = ~(np.abs(ref_norms / thresholds - 1.0) <= BAND)
    else:
        outside = np.ones(len(ref_flags), dtype=bool)
    mism = (gpu_flags != ref_flags) & outside
    assert not mism.any(), "%s: clip decision differs on tensors %s" % (name, np.nonzero(mism)[0][:10])


class Run:
    """One context + device state + a host mirror advanced by the oracle."""

    def __init__(self, workload, optimizer="adamw", device="cuda:0", mirror=True, **ctx_kw):
        self.w = workload
        self.device = device
        self.optimizer = B.ADAGC_OPT_ADAMW if optimizer == "adamw" else B.ADAGC_OPT_LION
        self.grad_dtype = B.ADAGC_GRAD_BF16 if workload.grad_dtype == torch.bfloat16 else B.ADAGC_GRAD_F32
        self.params, self.m, self.v, self.copies = workload.make_state(device, optimizer)
        self.gamma = torch.zeros(workload.n_tensors, dtype=torch.float32, device=device)
        self.ctx = B.AdaGC(workload.numels, self.optimizer, self.grad_dtype, workload.bf16_copy, **ctx_kw)
        if self.copies is not None:
            self.ctx.set_param_copies(self.copies)
        self.h = None
        if mirror:
            self.h_params = [to_numpy(t) for t in self.params]
            self.h_m = [to_numpy(t) for t in self.m]
            self.h_v = [to_numpy(t) for t in self.v] if self.v is not None else None
            self.h_copies = [to_numpy(t) for t in self.copies] if self.copies is not None else None
            self.h_gamma = np.zeros(workload.n_tensors, dtype=np.float32)

    def gpu_step(self, grads, hp, step):
        self.ctx.step(self.params, grads, self.m, self.v, self.gamma, hp, step)
        return self.ctx.get_norms()

    def oracle_step(self, grads_np, hp, step):
        ohp = oracle_hyper(hp, self.optimizer, self.grad_dtype)
        thr = ohp._step().lambda_rel * self.h_gamma.astype(np.float64)
        res = oracle.adagc_step(self.h_params, grads_np, self.h_m, self.h_v, self.h_gamma, ohp, step,
                                self.h_copies)
        return res + (thr,)

    def lion_exempt(self, i, grad_np, m_before, coef, hp, idx=None):
        """Elements (all, or those at `idx`) whose Lion interpolation is within 1e-6 relative of zero."""
        b1 = float(np.float32(hp.beta1))
        if idx is not None:
            grad_np, m_before = grad_np[idx], m_before[idx]
        g = widen_grad(grad_np).astype(np.float64)
        a = b1 * m_before.astype(np.float64)
        b = (1.0 - b1) * coef * g
        return np.abs(a + b) <= 1e-6 * (np.abs(a) + np.abs(b))

    def compare_state(self, name, exempt_theta=None):
        """Returns the number of stored values that are not bit-identical to the oracle's."""
        differ = 0
        for i in range(self.w.n_tensors):
            tag = "%s tensor %d (%s)" % (name, i, self.w.specs[i].name)
            ex = exempt_theta[i] if exempt_theta is not None else None
            gpu_theta = to_numpy(self.params[i])
            differ += assert_close(tag + " theta", gpu_theta, self.h_params[i], exempt=ex)
            differ += assert_close(tag + " m", to_numpy(self.m[i]), self.h_m[i])
            if self.v is not None:
                differ += assert_close(tag + " v", to_numpy(self.v[i]), self.h_v[i])
            if self.copies is not None:
                assert_bf16_copy(tag, to_numpy(self.copies[i]), gpu_theta, self.h_params[i], ex)
        return differ
