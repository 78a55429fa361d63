"""ctypes front end of the CPU oracle (``adagc_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
CPU-baseline leg of the benchmark.  Nothing in the GPU library or its Python
binding imports this package, and this package imports nothing of theirs.

All arrays are numpy arrays owned by the caller; float32 state arrays are
updated in place.  bf16 data travels as ``uint16`` bit patterns.
"""
import ctypes
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build
from .segments import enumerate_chunks  # noqa: F401  (re-export)

_lib = None

ADAMW = 0
LION = 1
GRAD_F32 = 0
GRAD_BF16 = 1
MODE_ADAGC = 0          # Alg. 1
MODE_GLOBALGC = 1       # Eq. 2 on every step
MODE_GLOBAL_ADAGC = 2   # one adaptive threshold for the whole model ("Ablation Study", Sec. 5.6)
MODE_ZCLIP = 3          # z-score clipping of the global norm (Table 2; appendix "Clipping Hyper-Parameters")
MODE_AGC = 4            # update clipping by the weights' l2 norm (Table 2)
MODE_CLIPPY = 5         # update clipping by the weights' l-infinity norm (Table 2)


class _OptHyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double)]


class _StepHyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double),
                ("lambda_rel", ctypes.c_double), ("ema_beta", ctypes.c_double),
                ("lambda_abs", ctypes.c_double), ("t_start", ctypes.c_int64),
                ("optimizer", ctypes.c_int32), ("grad_dtype", ctypes.c_int32),
                ("clip_mode", ctypes.c_int32), ("reserved", ctypes.c_int32), ("z_thres", ctypes.c_double)]


def _f32(x):
    """A hyper-parameter as the library receives it: a binary32 value, widened."""
    return float(np.float32(x))


@dataclass
class Hyper:
    """Hyper-parameters of Alg. 1.  Every value is rounded to binary32 first,
    because that is the type in which a caller hands them to the GPU library;
    the oracle then computes with the widened doubles."""
    lr: float = 3e-4
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1
    lambda_rel: float = 1.04      # default fixed in "Critical Hyperparameter Selection", Sec. 5.2
    ema_beta: float = 0.99        # same subsection
    lambda_abs: float = float("inf")
    t_start: int = 1
    optimizer: int = ADAMW
    grad_dtype: int = GRAD_F32
    clip_mode: int = MODE_ADAGC
    z_thres: float = 2.0          # ZClip only; appendix "Clipping Hyper-Parameters" (with alpha = ema_beta = 0.97)

    def _opt(self):
        return _OptHyper(_f32(self.lr), _f32(self.beta1), _f32(self.beta2), _f32(self.eps),
                         _f32(self.weight_decay))

    def _step(self):
        return _StepHyper(_f32(self.lr), _f32(self.beta1), _f32(self.beta2), _f32(self.eps),
                          _f32(self.weight_decay), _f32(self.lambda_rel), _f32(self.ema_beta),
                          _f32(self.lambda_abs), int(self.t_start), int(self.optimizer),
                          int(self.grad_dtype), int(self.clip_mode), 0, _f32(self.z_thres))


def _declare(L):
    vp, i64, dbl, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_double, ctypes.c_int
    L.oracle_num_threads.restype = i32
    L.oracle_num_threads.argtypes = []
    L.oracle_bf16_to_float.restype = ctypes.c_float
    L.oracle_bf16_to_float.argtypes = [ctypes.c_uint16]
    L.oracle_float_to_bf16_rne.restype = ctypes.c_uint16
    L.oracle_float_to_bf16_rne.argtypes = [ctypes.c_float]
    L.oracle_sum_squares.restype = dbl
    L.oracle_sum_squares.argtypes = [vp, i64, i32]
    L.oracle_l2_norm.restype = dbl
    L.oracle_l2_norm.argtypes = [vp, i64, i32]
    L.oracle_adagc_rule.restype = None
    L.oracle_adagc_rule.argtypes = [dbl, dbl, dbl, dbl, ctypes.POINTER(dbl),
                                    ctypes.POINTER(dbl), ctypes.POINTER(i32)]
    L.oracle_globalgc_coef.restype = dbl
    L.oracle_globalgc_coef.argtypes = [dbl, dbl]
    L.oracle_warmup_gamma.restype = dbl
    L.oracle_warmup_gamma.argtypes = [dbl, dbl, i32]
    L.oracle_zclip_rule.restype = None
    L.oracle_zclip_rule.argtypes = [dbl, dbl, dbl, dbl, dbl, ctypes.POINTER(dbl), ctypes.POINTER(dbl),
                                    ctypes.POINTER(dbl), ctypes.POINTER(i32)]
    L.oracle_zclip_gather.restype = None
    L.oracle_zclip_gather.argtypes = [dbl, dbl, dbl, dbl, i32, ctypes.POINTER(dbl), ctypes.POINTER(dbl)]
    L.oracle_agc_coef.restype = dbl
    L.oracle_agc_coef.argtypes = [dbl, dbl, dbl, ctypes.POINTER(i32)]
    L.oracle_clippy_coef.restype = dbl
    L.oracle_clippy_coef.argtypes = [dbl, dbl, dbl, dbl, dbl, ctypes.POINTER(i32)]
    L.oracle_direction_norms.restype = None
    L.oracle_direction_norms.argtypes = [vp, vp, vp, vp, i32, i64, ctypes.POINTER(_OptHyper), i32, i64,
                                         ctypes.POINTER(dbl), ctypes.POINTER(dbl), ctypes.POINTER(dbl),
                                         ctypes.POINTER(dbl)]
    L.oracle_adamw_update_clipped.restype = None
    L.oracle_adamw_update_clipped.argtypes = [vp, vp, vp, vp, i32, i64, dbl, ctypes.POINTER(_OptHyper), i64, vp]
    L.oracle_lion_update_clipped.restype = None
    L.oracle_lion_update_clipped.argtypes = [vp, vp, vp, i32, i64, dbl, ctypes.POINTER(_OptHyper), vp]
    L.oracle_adamw_update.restype = None
    L.oracle_adamw_update.argtypes = [vp, vp, vp, vp, i32, i64, dbl,
                                      ctypes.POINTER(_OptHyper), i64, vp]
    L.oracle_lion_update.restype = None
    L.oracle_lion_update.argtypes = [vp, vp, vp, i32, i64, dbl, ctypes.POINTER(_OptHyper), vp]
    L.oracle_state_norms.restype = None
    L.oracle_state_norms.argtypes = [vp, vp, vp, vp, i64, ctypes.POINTER(dbl), ctypes.POINTER(dbl),
                                     ctypes.POINTER(dbl)]
    L.oracle_adagc_step.restype = i32
    L.oracle_adagc_step.argtypes = [i64, vp, vp, vp, vp, vp, vp, vp,
                                    ctypes.POINTER(_StepHyper), i64, vp, vp, vp]
    return L


_lib_all_cores = None
_use_all_cores = False


def lib():
    """The oracle library in use: the one-thread build (the definition) unless all_cores() switched."""
    global _lib, _lib_all_cores
    if _use_all_cores:
        if _lib_all_cores is None:
            _lib_all_cores = _declare(ctypes.CDLL(_build.build(all_cores=True)))
        return _lib_all_cores
    if _lib is None:
        # ADAGC_ORACLE_LIB: a test may point at a deliberately broken build to show that the pins notice
        _lib = _declare(ctypes.CDLL(os.environ.get("ADAGC_ORACLE_LIB") or _build.build()))
    return _lib


class all_cores:
    """``with oracle.all_cores():`` runs the enclosed calls on the all-cores build of the same source
    (bit-identical theta / m / v / copies; sums of squares in another rounding order)."""

    def __enter__(self):
        global _use_all_cores
        self._saved = _use_all_cores
        _use_all_cores = True
        lib()
        return self

    def __exit__(self, *exc):
        global _use_all_cores
        _use_all_cores = self._saved
        return False


def num_threads():
    """Threads the per-element loops of the library in use run on."""
    return int(lib().oracle_num_threads())


def _grad_dtype(g):
    if g.dtype == np.float32:
        return GRAD_F32
    if g.dtype == np.uint16:
        return GRAD_BF16
    raise TypeError("gradient must be float32 or uint16 (bf16 bits), got %s" % g.dtype)


def _check(a, dtype, n=None):
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"] or a.ndim != 1:
        raise TypeError("need a contiguous 1-D %s array" % np.dtype(dtype).name)
    if n is not None and a.size != n:
        raise ValueError("array of %d elements where %d are needed" % (a.size, n))
    return a.ctypes.data


def bf16_to_float(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    f = lib().oracle_bf16_to_float
    return np.array([f(int(b)) for b in bits.ravel()], dtype=np.float32).reshape(bits.shape)


def float_to_bf16_rne(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    f = lib().oracle_float_to_bf16_rne
    return np.array([f(float(v)) for v in x.ravel()], dtype=np.uint16).reshape(x.shape)


def sum_squares(g):
    return lib().oracle_sum_squares(_check(g, g.dtype), g.size, _grad_dtype(g))


def l2_norm(g):
    return lib().oracle_l2_norm(_check(g, g.dtype), g.size, _grad_dtype(g))


def adagc_rule(norm, gamma_prev, lambda_rel, beta):
    h, gn, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
    lib().oracle_adagc_rule(norm, gamma_prev, lambda_rel, beta, ctypes.byref(h),
                            ctypes.byref(gn), ctypes.byref(c))
    return h.value, gn.value, bool(c.value)


def globalgc_coef(global_norm, lambda_abs):
    return lib().oracle_globalgc_coef(global_norm, lambda_abs)


def warmup_gamma(gamma_prev, clipped_norm, first_step):
    return lib().oracle_warmup_gamma(gamma_prev, clipped_norm, int(bool(first_step)))


def zclip_rule(norm, mu_prev, var_prev, alpha, z_thres):
    """(h, mu_new, var_new, clipped) of ZClip's z-score rule on one global norm."""
    h, mu, var, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
    lib().oracle_zclip_rule(norm, mu_prev, var_prev, alpha, z_thres, ctypes.byref(h), ctypes.byref(mu),
                            ctypes.byref(var), ctypes.byref(c))
    return h.value, mu.value, var.value, bool(c.value)


def zclip_gather(clipped_norm, mu_prev, var_prev, alpha, first_step):
    """(mu_new, var_new) on a step that only gathers ZClip's statistics."""
    mu, var = ctypes.c_double(), ctypes.c_double()
    lib().oracle_zclip_gather(clipped_norm, mu_prev, var_prev, alpha, int(bool(first_step)), ctypes.byref(mu),
                              ctypes.byref(var))
    return mu.value, var.value


def adamw_update(theta, m, v, g, h, hyper, t, theta_bf16=None):
    n = theta.size
    oh = hyper._opt()
    lib().oracle_adamw_update(_check(theta, np.float32), _check(m, np.float32, n),
                              _check(v, np.float32, n), _check(g, g.dtype, n), _grad_dtype(g),
                              n, float(h), ctypes.byref(oh), int(t),
                              None if theta_bf16 is None else _check(theta_bf16, np.uint16, n))


def lion_update(theta, m, g, h, hyper, theta_bf16=None):
    n = theta.size
    oh = hyper._opt()
    lib().oracle_lion_update(_check(theta, np.float32), _check(m, np.float32, n),
                             _check(g, g.dtype, n), _grad_dtype(g), n, float(h),
                             ctypes.byref(oh),
                             None if theta_bf16 is None else _check(theta_bf16, np.uint16, n))


def agc_coef(theta_norm, delta_norm, lambda_rel):
    """(coefficient, clipped) of Table 2's AGC row."""
    c = ctypes.c_int()
    return lib().oracle_agc_coef(theta_norm, delta_norm, lambda_rel, ctypes.byref(c)), bool(c.value)


def clippy_coef(theta_inf, delta_inf, lambda_rel, lambda_abs, lr):
    """(coefficient, clipped) of Table 2's Clippy row."""
    c = ctypes.c_int()
    return lib().oracle_clippy_coef(theta_inf, delta_inf, lambda_rel, lambda_abs, lr, ctypes.byref(c)), bool(c.value)


def direction_norms(theta, m, v, g, hyper, t):
    """(||theta||_2, ||Delta||_2, ||theta||_inf, ||Delta||_inf) for the direction this step's unclipped
    gradient produces (AdamW: mhat/(sqrt(vhat)+eps); Lion, v=None: the sign of the interpolation)."""
    n = theta.size
    oh = hyper._opt()
    out = [ctypes.c_double() for _ in range(4)]
    lib().oracle_direction_norms(_check(theta, np.float32), _check(m, np.float32, n),
                                 None if v is None else _check(v, np.float32, n), _check(g, g.dtype, n),
                                 _grad_dtype(g), n, ctypes.byref(oh), int(hyper.optimizer), int(t),
                                 *[ctypes.byref(x) for x in out])
    return tuple(x.value for x in out)


def adamw_update_clipped(theta, m, v, g, update_coef, hyper, t, theta_bf16=None):
    n = theta.size
    oh = hyper._opt()
    lib().oracle_adamw_update_clipped(_check(theta, np.float32), _check(m, np.float32, n),
                                      _check(v, np.float32, n), _check(g, g.dtype, n), _grad_dtype(g),
                                      n, float(update_coef), ctypes.byref(oh), int(t),
                                      None if theta_bf16 is None else _check(theta_bf16, np.uint16, n))


def lion_update_clipped(theta, m, g, update_coef, hyper, theta_bf16=None):
    n = theta.size
    oh = hyper._opt()
    lib().oracle_lion_update_clipped(_check(theta, np.float32), _check(m, np.float32, n),
                                     _check(g, g.dtype, n), _grad_dtype(g), n, float(update_coef),
                                     ctypes.byref(oh),
                                     None if theta_bf16 is None else _check(theta_bf16, np.uint16, n))


def state_norms(theta_before, theta_after, m, v=None):
    """(||m||, ||v||, ||theta_after - theta_before||) of one tensor, from the stored float32 values."""
    n = theta_after.size
    a, b, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    lib().oracle_state_norms(_check(theta_before, np.float32, n), _check(theta_after, np.float32, n),
                             _check(m, np.float32, n), None if v is None else _check(v, np.float32, n), n,
                             ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    return a.value, b.value, c.value


def adagc_step(theta, grad, m, v, gamma, hyper, step, theta_bf16=None):
    """One pass of the body of Alg. 1 over a list of tensors.

    theta, grad, m, v (None for Lion), theta_bf16 (or None): lists of 1-D arrays.
    gamma: float32 array, one entry per tensor, updated in place (MODE_ZCLIP: entries 0 and 1 hold the
    mean and the variance of the global norm, so a one-tensor list needs two entries).
    Returns (norms float64[n], coefs float64[n], clipped uint8[n]).
    """
    n = len(theta)
    gd = _grad_dtype(grad[0])
    if gd != hyper.grad_dtype:
        raise ValueError("gradient dtype does not match hyper.grad_dtype")
    numel = np.array([t.size for t in theta], dtype=np.int64)

    def ptrs(arrs, dtype):
        out = (ctypes.c_void_p * n)()
        for i, a in enumerate(arrs):
            out[i] = _check(a, dtype, int(numel[i]))
        return out

    p_theta = ptrs(theta, np.float32)
    p_grad = ptrs(grad, grad[0].dtype)
    p_m = ptrs(m, np.float32)
    p_v = ptrs(v, np.float32) if v is not None else None
    p_c = ptrs(theta_bf16, np.uint16) if theta_bf16 is not None else None
    norms = np.zeros(n, dtype=np.float64)
    coefs = np.zeros(n, dtype=np.float64)
    clipped = np.zeros(n, dtype=np.uint8)
    sh = hyper._step()
    rc = lib().oracle_adagc_step(n, numel.ctypes.data, p_theta, p_grad, p_m, p_v, p_c,
                                 _check(gamma, np.float32, max(n, 2) if hyper.clip_mode == MODE_ZCLIP else n),
                                 ctypes.byref(sh), int(step),
                                 norms.ctypes.data, coefs.ctypes.data, clipped.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_adagc_step rejected its arguments")
    return norms, coefs, clipped
