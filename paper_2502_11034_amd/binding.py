"""ctypes binding of libadagc: the same entry points as include/adagc.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels; if the
library is missing this module raises instead of falling back to anything else.

PyTorch is used by callers for device memory and streams; this module only reads
``tensor.data_ptr()``.
"""
import ctypes
import os

import numpy as np

from . import build as _build

ADAGC_OK = 0
ADAGC_ERR_INVALID_ARG = -1
ADAGC_ERR_OOM = -2
ADAGC_ERR_HIP = -3
ADAGC_ERR_TOO_LARGE = -4
ADAGC_ERR_STATE = -5

ADAGC_OPT_ADAMW, ADAGC_OPT_LION, ADAGC_OPT_MUON = 0, 1, 2
ADAGC_GRAD_F32, ADAGC_GRAD_BF16 = 0, 1
ADAGC_MODE_ADAGC, ADAGC_MODE_GLOBALGC, ADAGC_MODE_GLOBAL_ADAGC, ADAGC_MODE_ZCLIP = 0, 1, 2, 3
ADAGC_MODE_AGC, ADAGC_MODE_CLIPPY = 4, 5

EXPORTS = [
    "adagc_chunk_elems", "adagc_build_segment_table", "adagc_build_visiting_order", "adagc_create", "adagc_destroy",
    "adagc_set_param_copies", "adagc_step", "adagc_step_graph", "adagc_step_static", "adagc_get_norms", "adagc_get_state_norms", "adagc_num_tensors",
    "adagc_num_chunks", "adagc_get_segment_table", "adagc_profile_begin", "adagc_profile_end", "adagc_muon_gemm_nt", "adagc_muon_gemm_nt_batched", "adagc_muon_attach",
    "adagc_muon_workspace_bytes", "adagc_muon_step",
    "adagc_strerror",
]


class adagc_tensor_desc(ctypes.Structure):
    _fields_ = [("numel", ctypes.c_int64), ("flags", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class adagc_config(ctypes.Structure):
    _fields_ = [("optimizer", ctypes.c_int32), ("grad_dtype", ctypes.c_int32),
                ("has_bf16_param_copy", ctypes.c_int32), ("telemetry", ctypes.c_int32),
                ("grid_blocks", ctypes.c_int32),
                ("unroll", ctypes.c_int32), ("nontemporal", ctypes.c_int32), ("schedule", ctypes.c_int32),
                ("update_split", ctypes.c_int32), ("schedule_run", ctypes.c_int32),
                ("update_clipping", ctypes.c_int32)]


class adagc_hyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("lambda_rel", ctypes.c_float), ("ema_beta", ctypes.c_float),
                ("lambda_abs", ctypes.c_float), ("t_start", ctypes.c_int32), ("clip_mode", ctypes.c_int32),
                ("z_thres", ctypes.c_float)]


class adagc_matrix_shape(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64)]


class adagc_muon_hyper(ctypes.Structure):
    _fields_ = [("momentum", ctypes.c_float), ("nesterov", ctypes.c_int32), ("ns_steps", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class adagc_step_params(ctypes.Structure):
    _fields_ = [("hp", adagc_hyper), ("step", ctypes.c_int64)]


class AdagcError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, strerror(code), code))


_lib = None


def lib():
    """Open libadagc.so (built in-tree).  Raises if it is not there: there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB
    if not os.path.exists(path):
        raise RuntimeError("libadagc.so is not built (%s); run __graft_entry__.build() or "
                           "python -m paper_2502_11034_amd.build" % path)
    L = ctypes.CDLL(path)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    L.adagc_chunk_elems.restype = i64
    L.adagc_chunk_elems.argtypes = []
    L.adagc_build_visiting_order.restype = ctypes.c_int
    L.adagc_build_visiting_order.argtypes = [i64, ctypes.c_int32, ctypes.c_int32, vp]
    L.adagc_build_segment_table.restype = ctypes.c_int
    L.adagc_build_segment_table.argtypes = [vp, i64, i64, vp, vp, vp, i64, ctypes.POINTER(i64)]
    L.adagc_create.restype = ctypes.c_int
    L.adagc_create.argtypes = [ctypes.POINTER(vp), vp, i64, ctypes.POINTER(adagc_config)]
    L.adagc_destroy.restype = None
    L.adagc_destroy.argtypes = [vp]
    L.adagc_set_param_copies.restype = ctypes.c_int
    L.adagc_set_param_copies.argtypes = [vp, vp]
    L.adagc_step.restype = ctypes.c_int
    L.adagc_step.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.POINTER(adagc_hyper), i64, vp]
    L.adagc_step_graph.restype = ctypes.c_int
    L.adagc_step_graph.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    L.adagc_step_static.restype = ctypes.c_int
    L.adagc_step_static.argtypes = [vp, i64, ctypes.POINTER(adagc_config), vp, vp, vp, vp, vp, vp,
                                    ctypes.POINTER(adagc_hyper), i64, vp, vp, vp, vp]
    L.adagc_get_norms.restype = ctypes.c_int
    L.adagc_get_norms.argtypes = [vp, vp, vp, vp, i64, vp]
    L.adagc_get_state_norms.restype = ctypes.c_int
    L.adagc_get_state_norms.argtypes = [vp, vp, vp, vp, i64, vp]
    L.adagc_num_tensors.restype = i64
    L.adagc_num_tensors.argtypes = [vp]
    L.adagc_num_chunks.restype = i64
    L.adagc_num_chunks.argtypes = [vp]
    L.adagc_get_segment_table.restype = ctypes.c_int
    L.adagc_get_segment_table.argtypes = [vp, vp, vp, vp]
    L.adagc_profile_begin.restype = ctypes.c_int
    L.adagc_profile_begin.argtypes = [vp, i32]
    L.adagc_profile_end.restype = ctypes.c_int
    L.adagc_profile_end.argtypes = [vp, vp, ctypes.POINTER(i32)]
    L.adagc_muon_attach.restype = ctypes.c_int
    L.adagc_muon_attach.argtypes = [vp, vp]
    L.adagc_muon_step.restype = ctypes.c_int
    L.adagc_muon_step.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(adagc_hyper), ctypes.POINTER(adagc_muon_hyper), i64, vp]
    L.adagc_muon_gemm_nt.restype = ctypes.c_int
    L.adagc_muon_gemm_nt.argtypes = [vp, i64, vp, i64, i64, i64, i64, ctypes.c_float, ctypes.c_float, vp, i64, vp, i64,
                                     vp, i64, i32, vp]
    L.adagc_muon_gemm_nt_batched.restype = ctypes.c_int
    L.adagc_muon_gemm_nt_batched.argtypes = [vp, i64, vp, i64, i64, i64, i64, ctypes.c_float, ctypes.c_float, vp, i64, vp, i64,
                                             vp, i64, i32, i64, vp, vp]
    L.adagc_muon_workspace_bytes.restype = ctypes.c_int64
    L.adagc_muon_workspace_bytes.argtypes = [vp]
    L.adagc_strerror.restype = ctypes.c_char_p
    L.adagc_strerror.argtypes = [ctypes.c_int]
    _lib = L
    return L


def strerror(code):
    return lib().adagc_strerror(int(code)).decode()


def _check(rc, where):
    if rc != ADAGC_OK:
        raise AdagcError(rc, where)


def _descs(numels):
    arr = (adagc_tensor_desc * len(numels))()
    for i, n in enumerate(numels):
        arr[i].numel = int(n)
    return arr


def ptr_array(tensors):
    """Host array of device pointers from a list of tensors (returned as is if already one)."""
    if isinstance(tensors, ctypes.Array):
        return tensors
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr() if hasattr(t, "data_ptr") else int(t)
    return arr


def adagc_chunk_elems():
    return int(lib().adagc_chunk_elems())


def adagc_build_segment_table(numels, chunk_elems=None):
    """Host-only.  Returns (chunk_begin int64[n+1], chunk_tensor uint32[c], chunk_index uint32[c])."""
    L = lib()
    n = len(numels)
    chunk_elems = adagc_chunk_elems() if chunk_elems is None else int(chunk_elems)
    descs = _descs(numels) if n else None
    begin = np.zeros(n + 1, dtype=np.int64)
    total = ctypes.c_int64(0)
    _check(L.adagc_build_segment_table(ctypes.cast(descs, ctypes.c_void_p) if n else None, n, chunk_elems,
                                       begin.ctypes.data, None, None, 0, ctypes.byref(total)),
           "adagc_build_segment_table")
    c = total.value
    tensor = np.zeros(c, dtype=np.uint32)
    index = np.zeros(c, dtype=np.uint32)
    _check(L.adagc_build_segment_table(ctypes.cast(descs, ctypes.c_void_p), n, chunk_elems,
                                       begin.ctypes.data, tensor.ctypes.data, index.ctypes.data, c,
                                       ctypes.byref(total)),
           "adagc_build_segment_table")
    return begin, tensor, index


def step_params_bytes(hyper, step):
    """The bytes of an adagc_step_params, ready to be copied into device memory."""
    return bytes(adagc_step_params(hyper, int(step)))


def adagc_build_visiting_order(n_chunks, parts=2, run=8):
    """Host-only.  Returns the visiting order, uint32[n_chunks]."""
    order = np.zeros(max(int(n_chunks), 0), dtype=np.uint32)
    _check(lib().adagc_build_visiting_order(int(n_chunks), int(parts), int(run),
                                            order.ctypes.data if order.size else None),
           "adagc_build_visiting_order")
    return order


def adagc_muon_gemm_nt(P, Q, alpha=1.0, beta=0.0, Dt=None, C=None, Ct=None, stream=None, symmetric=False):
    """adagc_muon_gemm_nt on 2-D bf16 device tensors (row-major, possibly with a leading dimension larger than
    the row length): C = bf16(alpha P Q^T + beta D), D passed as its transpose Dt."""
    M, K = P.shape
    N = Q.shape[0]
    ld = lambda t: t.stride(0) if t is not None else 0
    dp = lambda t: t.data_ptr() if t is not None else None
    _check(lib().adagc_muon_gemm_nt(P.data_ptr(), ld(P), Q.data_ptr(), ld(Q), M, N, K, float(alpha), float(beta), dp(Dt),
                                    ld(Dt), dp(C), ld(C), dp(Ct), ld(Ct), int(bool(symmetric)),
                                    ctypes.c_void_p(stream) if stream else None),
           "adagc_muon_gemm_nt")


def adagc_muon_gemm_nt_batched(P, Q, alpha=1.0, beta=0.0, Dt=None, C=None, Ct=None, stream=None, symmetric=False):
    """adagc_muon_gemm_nt_batched on 3-D bf16 device tensors [batch, rows, cols]: matrix z of every array is its [z]."""
    batch, M, K = P.shape
    N = Q.shape[1]
    ld = lambda t: t.stride(1) if t is not None else 0
    dp = lambda t: t.data_ptr() if t is not None else None
    strides = (ctypes.c_int64 * 5)(*[t.stride(0) if t is not None else 0 for t in (P, Q, Dt, C, Ct)])
    _check(lib().adagc_muon_gemm_nt_batched(P.data_ptr(), ld(P), Q.data_ptr(), ld(Q), M, N, K, float(alpha), float(beta), dp(Dt),
                                            ld(Dt), dp(C), ld(C), dp(Ct), ld(Ct), int(bool(symmetric)), int(batch), strides,
                                            ctypes.c_void_p(stream) if stream else None),
           "adagc_muon_gemm_nt_batched")


ADAGC_STATIC_MAX_TENSORS = 32768
ADAGC_STATIC_MAX_CHUNKS = 524288


def adagc_step_static(numels, params, grads, exp_avg, exp_avg_sq, ema_norms, hyper, step, optimizer=ADAGC_OPT_ADAMW,
                      grad_dtype=ADAGC_GRAD_F32, params_bf16=None, out_norms=None, out_coefs=None, out_clipped=None,
                      stream=None):
    """adagc_step_static: the step without a context and without any allocation on the GPU side.
    out_*: device tensors (or None).  Raises AdagcError on a non-zero return code."""
    cfg = adagc_config(int(optimizer), int(grad_dtype), int(params_bf16 is not None), 0, 0, 0, 0, 0, 0, 0, 0)
    descs = _descs([int(n) for n in numels])
    p, g, m = (ptr_array(x) for x in (params, grads, exp_avg))
    v = ptr_array(exp_avg_sq) if exp_avg_sq is not None else None
    c = ptr_array(params_bf16) if params_bf16 is not None else None
    dp = lambda t: t.data_ptr() if t is not None else None
    _check(lib().adagc_step_static(ctypes.cast(descs, ctypes.c_void_p), len(numels), ctypes.byref(cfg), p, g, m, v, c,
                                   ema_norms.data_ptr(), ctypes.byref(hyper), int(step), dp(out_norms),
                                   dp(out_coefs), dp(out_clipped), ctypes.c_void_p(stream) if stream else None),
           "adagc_step_static")


class AdaGC:
    """Owner of one adagc_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, numels, optimizer=ADAGC_OPT_ADAMW, grad_dtype=ADAGC_GRAD_F32,
                 has_bf16_param_copy=False, grid_blocks=0, unroll=0, nontemporal=0, schedule=0, telemetry=False,
                 update_split=0, schedule_run=0, update_clipping=False):
        L = lib()
        self._ctx = ctypes.c_void_p(None)
        self.n_tensors = len(numels)
        self.numels = [int(n) for n in numels]
        cfg = adagc_config(int(optimizer), int(grad_dtype), int(bool(has_bf16_param_copy)), int(bool(telemetry)),
                           int(grid_blocks), int(unroll), int(nontemporal), int(schedule), int(update_split), int(schedule_run),
                           int(bool(update_clipping)))
        descs = _descs(self.numels)
        _check(L.adagc_create(ctypes.byref(self._ctx), ctypes.cast(descs, ctypes.c_void_p), self.n_tensors,
                              ctypes.byref(cfg)), "adagc_create")
        self.optimizer = int(optimizer)

    # -- adagc_destroy
    def close(self):
        ctx = getattr(self, "_ctx", None)
        if ctx is not None and ctx.value and _lib is not None:     # _lib is gone at interpreter shutdown
            _lib.adagc_destroy(ctx)
            self._ctx = ctypes.c_void_p(None)

    __del__ = close

    # -- adagc_set_param_copies
    def set_param_copies(self, copies):
        _check(lib().adagc_set_param_copies(self._ctx, ptr_array(copies)), "adagc_set_param_copies")

    # -- adagc_step
    def step(self, params, grads, exp_avg, exp_avg_sq, ema_norms, hyper, step, stream=None):
        """params/grads/exp_avg/exp_avg_sq: lists of device tensors, or pointer arrays made once with
        ptr_array() (saves re-marshalling long lists every step); ema_norms: device fp32[n];
        hyper: adagc_hyper; stream: raw hipStream_t handle (int) or None for the default stream."""
        p, g, m = (ptr_array(x) for x in (params, grads, exp_avg))
        v = ptr_array(exp_avg_sq) if exp_avg_sq is not None else None
        _check(lib().adagc_step(self._ctx, p, g, m, v, ema_norms.data_ptr(), ctypes.byref(hyper), int(step),
                                ctypes.c_void_p(stream) if stream else None), "adagc_step")

    # -- adagc_muon_attach / adagc_muon_step
    def muon_attach(self, shapes):
        arr = (adagc_matrix_shape * len(shapes))()
        for i, (r, c) in enumerate(shapes):
            arr[i].rows, arr[i].cols = int(r), int(c)
        _check(lib().adagc_muon_attach(self._ctx, ctypes.cast(arr, ctypes.c_void_p)), "adagc_muon_attach")

    def muon_workspace_bytes(self):
        return int(lib().adagc_muon_workspace_bytes(self._ctx))

    def muon_step(self, params, grads, momentum, ema_norms, hyper, muon_hyper, step, stream=None):
        p, g, m = (ptr_array(x) for x in (params, grads, momentum))
        _check(lib().adagc_muon_step(self._ctx, p, g, m, ema_norms.data_ptr(), ctypes.byref(hyper), ctypes.byref(muon_hyper),
                                     int(step), ctypes.c_void_p(stream) if stream else None), "adagc_muon_step")

    # -- adagc_step_graph
    def step_graph(self, params, grads, exp_avg, exp_avg_sq, ema_norms, step_params, stream=None):
        """As step(), with hyper-parameters and step number read on the GPU from `step_params`: a device
        tensor of sizeof(adagc_step_params) = 56 bytes holding an adagc_step_params (see step_params_bytes)."""
        p, g, m = (ptr_array(x) for x in (params, grads, exp_avg))
        v = ptr_array(exp_avg_sq) if exp_avg_sq is not None else None
        _check(lib().adagc_step_graph(self._ctx, p, g, m, v, ema_norms.data_ptr(), step_params.data_ptr(),
                                      ctypes.c_void_p(stream) if stream else None), "adagc_step_graph")

    # -- adagc_get_norms
    def get_norms(self, stream=None):
        n = self.n_tensors
        norms = np.zeros(n, dtype=np.float32)
        coefs = np.zeros(n, dtype=np.float32)
        clipped = np.zeros(n, dtype=np.uint8)
        _check(lib().adagc_get_norms(self._ctx, norms.ctypes.data, coefs.ctypes.data, clipped.ctypes.data, n,
                                     ctypes.c_void_p(stream) if stream else None), "adagc_get_norms")
        return norms, coefs, clipped

    # -- adagc_get_state_norms
    def get_state_norms(self, stream=None):
        n = self.n_tensors
        out = [np.zeros(n, dtype=np.float32) for _ in range(3)]
        _check(lib().adagc_get_state_norms(self._ctx, out[0].ctypes.data, out[1].ctypes.data, out[2].ctypes.data,
                                           n, ctypes.c_void_p(stream) if stream else None), "adagc_get_state_norms")
        return tuple(out)

    # -- adagc_num_chunks / adagc_get_segment_table
    def num_chunks(self):
        return int(lib().adagc_num_chunks(self._ctx))

    def get_segment_table(self):
        c = self.num_chunks()
        begin = np.zeros(self.n_tensors + 1, dtype=np.int64)
        tensor = np.zeros(c, dtype=np.uint32)
        index = np.zeros(c, dtype=np.uint32)
        _check(lib().adagc_get_segment_table(self._ctx, begin.ctypes.data, tensor.ctypes.data,
                                             index.ctypes.data), "adagc_get_segment_table")
        return begin, tensor, index

    # -- adagc_profile_begin / adagc_profile_end
    def profile_begin(self, max_steps):
        self._prof_cap = int(max_steps)
        _check(lib().adagc_profile_begin(self._ctx, int(max_steps)), "adagc_profile_begin")

    def profile_end(self):
        ms = np.zeros(3 * self._prof_cap, dtype=np.float32)
        n = ctypes.c_int32(0)
        _check(lib().adagc_profile_end(self._ctx, ms.ctypes.data, ctypes.byref(n)), "adagc_profile_end")
        return ms[:3 * n.value].reshape(n.value, 3).copy()


def make_muon_hyper(momentum=0.95, nesterov=True, ns_steps=5):
    return adagc_muon_hyper(momentum, int(bool(nesterov)), int(ns_steps), 0)


def make_hyper(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, lambda_rel=1.04,
               ema_beta=0.99, lambda_abs=float("inf"), t_start=1, clip_mode=ADAGC_MODE_ADAGC, z_thres=2.0):
    return adagc_hyper(lr, beta1, beta2, eps, weight_decay, lambda_rel, ema_beta, lambda_abs, int(t_start),
                       int(clip_mode), z_thres)
