"""Thin Python binding of libmpq (ctypes): the same calls as ``include/mpq.h``, same names.

Argument marshalling only -- every step of the path runs in the HIP kernels of ``libmpq.so``.
PyTorch is used for device memory and streams, nothing else.  There is no CPU fallback: if the
library cannot be loaded (or built), importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

from . import build as _build

PER_TENSOR, PER_ROW, PER_COL = 0, 1, 2
OK = 0
ERR_NULL, ERR_SHAPE, ERR_BITS, ERR_ALIGN, ERR_WORKSPACE, ERR_GRAN, ERR_HIP, ERR_TOO_LARGE = 1, 2, 3, 4, 5, 6, 7, 8
NOALLOC_SCRATCH_BYTES = 4 << 20

EXPORTS = [
    "mpq_strerror", "mpq_last_hip_error", "mpq_version", "mpq_init", "mpq_calibrate_absmax_workspace_bytes",
    "mpq_calibrate_absmax",
    "mpq_scale_from_absmax", "mpq_fake_quant", "mpq_quant_error_workspace_bytes",
    "mpq_quant_error", "mpq_quant_error_noalloc", "mpq_noise_inject",
    "mpq_eqe", "mpq_eqe_channels", "mpq_hutchinson_trace", "mpq_latency_estimate", "mpq_model_size_bytes",
    "mpq_sweep_plan_bytes", "mpq_sweep_plan_build", "mpq_calibrate_absmax_batch",
    "mpq_calibrate_quant_error_rows_batch",
    "mpq_quant_error_batch_workspace_bytes", "mpq_quant_error_batch", "mpq_qgemm_workspace_bytes", "mpq_qgemm",
    "mpq_sse_pair_workspace_bytes", "mpq_sse_pair", "mpq_qgemm_score_workspace_bytes", "mpq_qgemm_score",
    "mpq_search_bisection", "mpq_search_greedy", "mpq_noise_inject_sweep",
    "mpq_fake_quant_scales", "mpq_scale_grad_workspace_bytes", "mpq_scale_grad", "mpq_scale_sgd_step", "mpq_qgemm_act", "mpq_qgemm_act_codes",
    "mpq_diag_mfma_operand_bytes", "mpq_diag_mfma_rate", "mpq_diag_sweep_alu_rate", "mpq_fake_quant_step", "mpq_stack_evaluate_workspace_bytes", "mpq_stack_evaluate", "mpq_rademacher", "mpq_hutchinson_quad_workspace_bytes", "mpq_hutchinson_quad", "mpq_hutchinson_quad_signs",
]

ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2
EVAL_FN = C.CFUNCTYPE(C.c_double, C.POINTER(C.c_int), C.c_int, C.c_void_p)
SEARCH_ENSURE_TARGET = 1

_lib = None


class MpqError(RuntimeError):
    def __init__(self, status: int, call: str):
        self.status = status
        msg = lib().mpq_strerror(status).decode()
        if status == ERR_HIP:
            msg += " (hipError %d)" % lib().mpq_last_hip_error()
        super().__init__("%s: %s" % (call, msg))


def lib():
    """Loads libmpq.so (built in-tree); builds it first only if no built library exists."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build_lib()
        # torch ships its own HIP runtime; whichever copy is loaded first serves the whole process,
        # and device buffers made by torch must belong to the runtime that launches the kernels
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(path)
        vp, i64, ci, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
        L.mpq_strerror.restype = C.c_char_p
        L.mpq_strerror.argtypes = [ci]
        L.mpq_last_hip_error.restype = ci
        L.mpq_version.restype = ci
        L.mpq_init.restype = ci
        L.mpq_init.argtypes = []
        L.mpq_calibrate_absmax_workspace_bytes.restype = sz
        L.mpq_calibrate_absmax_workspace_bytes.argtypes = [i64, i64, ci]
        L.mpq_calibrate_absmax.argtypes = [vp, i64, i64, ci, ci, vp, vp, sz, vp]
        L.mpq_scale_from_absmax.argtypes = [vp, i64, ci, vp, vp]
        L.mpq_fake_quant.argtypes = [vp, i64, i64, ci, vp, ci, vp, vp, vp, vp]
        L.mpq_quant_error_workspace_bytes.restype = sz
        L.mpq_quant_error_workspace_bytes.argtypes = [i64, i64, ci, ci, ci]
        L.mpq_quant_error.argtypes = [vp, i64, i64, ci, vp, ci, ci, vp, vp, sz, vp]
        L.mpq_quant_error_noalloc.argtypes = [vp, i64, i64, ci, vp, ci, ci, vp, vp]
        L.mpq_eqe.restype = C.c_double
        L.mpq_eqe.argtypes = [C.c_double, i64, C.c_double]
        L.mpq_eqe_channels.argtypes = [vp, vp, i64, ci, i64, vp]
        L.mpq_hutchinson_trace.argtypes = [vp, i64, i64, vp, vp]
        L.mpq_latency_estimate.argtypes = [vp, ci, ci, vp, vp]
        L.mpq_model_size_bytes.argtypes = [vp, vp, ci, vp]
        L.mpq_sweep_plan_bytes.restype = sz
        L.mpq_sweep_plan_bytes.argtypes = [vp, ci]
        L.mpq_sweep_plan_build.argtypes = [vp, ci, vp, sz]
        L.mpq_calibrate_absmax_batch.argtypes = [vp, vp, vp]
        L.mpq_calibrate_quant_error_rows_batch.argtypes = [vp, vp, ci, ci, vp]
        L.mpq_quant_error_batch_workspace_bytes.restype = sz
        L.mpq_quant_error_batch_workspace_bytes.argtypes = [vp, ci, ci, ci]
        L.mpq_quant_error_batch.argtypes = [vp, vp, ci, ci, ci, vp, sz, vp]
        L.mpq_noise_inject.argtypes = [vp, i64, i64, ci, vp, ci, C.c_float, C.c_uint64, C.c_uint64, vp, vp]
        L.mpq_noise_inject_sweep.argtypes = [vp, i64, i64, ci, vp, ci, ci, C.c_float, C.c_uint64, C.c_uint64, vp, i64, vp]
        L.mpq_fake_quant_scales.argtypes = [vp, i64, i64, ci, vp, vp, ci, vp, vp, vp]
        L.mpq_scale_grad_workspace_bytes.restype = sz
        L.mpq_scale_grad_workspace_bytes.argtypes = [i64, i64, ci]
        L.mpq_scale_grad.argtypes = [vp, i64, i64, ci, vp, vp, ci, vp, vp, vp, vp, vp, sz, vp]
        L.mpq_scale_sgd_step.argtypes = [vp, vp, vp, vp, i64, C.c_double, vp]
        L.mpq_qgemm_act.argtypes = [vp, vp, ci, i64, i64, i64, vp, vp, ci, ci, vp, vp, ci, vp]
        L.mpq_qgemm_act_codes.argtypes = [vp, vp, ci, i64, i64, i64, vp, vp, ci, ci, vp, ci, vp, vp]
        L.mpq_diag_mfma_operand_bytes.argtypes = []
        L.mpq_diag_mfma_operand_bytes.restype = C.c_size_t
        L.mpq_diag_mfma_rate.argtypes = [vp, C.c_size_t, ci, vp, C.POINTER(C.c_double), vp]
        L.mpq_diag_sweep_alu_rate.argtypes = [ci, vp, C.POINTER(C.c_double), vp]
        L.mpq_fake_quant_step.argtypes = [vp, i64, i64, vp, ci, vp, vp, vp, vp, vp]
        L.mpq_stack_evaluate_workspace_bytes.argtypes = [vp, ci, i64]
        L.mpq_stack_evaluate_workspace_bytes.restype = C.c_size_t
        L.mpq_stack_evaluate.argtypes = [vp, ci, i64, vp, ci, ci, ci, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.mpq_rademacher.argtypes = [C.c_uint64, C.c_uint64, i64, i64, vp, vp]
        L.mpq_hutchinson_quad_workspace_bytes.argtypes = [i64, i64, i64]
        L.mpq_hutchinson_quad_workspace_bytes.restype = C.c_size_t
        L.mpq_hutchinson_quad.argtypes = [vp, i64, i64, vp, i64, vp, vp, C.c_size_t, vp]
        L.mpq_hutchinson_quad_signs.argtypes = [vp, i64, i64, C.c_uint64, C.c_uint64, i64, vp, vp, C.c_size_t, vp]
        L.mpq_qgemm_workspace_bytes.restype = sz
        L.mpq_qgemm_workspace_bytes.argtypes = [i64, i64, i64, ci]
        L.mpq_qgemm.argtypes = [vp, vp, ci, i64, i64, i64, vp, vp, ci, vp, vp, vp, sz, vp]
        L.mpq_sse_pair_workspace_bytes.restype = sz
        L.mpq_sse_pair_workspace_bytes.argtypes = [i64]
        L.mpq_sse_pair.argtypes = [vp, vp, i64, vp, vp, sz, vp]
        L.mpq_qgemm_score_workspace_bytes.restype = sz
        L.mpq_qgemm_score_workspace_bytes.argtypes = [i64, i64, i64, ci]
        L.mpq_qgemm_score.argtypes = [vp, vp, ci, i64, i64, i64, vp, vp, ci, vp, vp, vp, vp, sz, vp]
        for f in (L.mpq_search_bisection, L.mpq_search_greedy):
            f.argtypes = [vp, ci, vp, ci, C.c_double, ci, EVAL_FN, vp, vp, vp]
        for name in EXPORTS:
            getattr(L, name)  # raises AttributeError if the library lacks a declared symbol
        _lib = L
    return _lib


def init():
    """Configures every kernel variant that needs it on the current device (see mpq_init)."""
    _check(lib().mpq_init(), "mpq_init")


def _check(status: int, call: str):
    if status != OK:
        raise MpqError(status, call)


# ---------------------------------------------------------------------------------------------
# torch plumbing (device buffers and the current stream)
def _torch():
    import torch
    return torch


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return _torch().cuda.current_stream().cuda_stream


def _dev2d(x, dtype):
    torch = _torch()
    if not x.is_cuda:
        raise ValueError("libmpq works on device tensors")
    if x.dim() != 2 or x.dtype != dtype or not x.is_contiguous():
        raise ValueError("expected a contiguous 2-D %s tensor" % dtype)
    return x


def _nch(gran, rows, cols):
    return {PER_TENSOR: 1, PER_ROW: rows, PER_COL: cols}[gran]


class Workspace:
    """A growable device scratch buffer handed to the calls that need one."""

    def __init__(self):
        self.buf = None

    def get(self, nbytes: int):
        torch = _torch()
        if nbytes == 0:
            return None, 0
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = torch.empty(max(nbytes, 1 << 16), dtype=torch.uint8, device="cuda")
        return self.buf.data_ptr(), self.buf.numel()


_default_ws = Workspace()


# ---------------------------------------------------------------------------------------------
def calibrate_absmax_workspace_bytes(rows, cols, gran=PER_TENSOR) -> int:
    return int(lib().mpq_calibrate_absmax_workspace_bytes(rows, cols, gran))


def calibrate_absmax(x, gran=PER_TENSOR, out=None, accumulate=False, ws: "Workspace" = None):
    torch = _torch()
    x = _dev2d(x, torch.float32)
    rows, cols = x.shape
    if out is None:
        if accumulate:
            raise ValueError("accumulate needs the running absmax in `out`")
        out = torch.empty(_nch(gran, rows, cols), dtype=torch.float32, device=x.device)
    wp, wn = (ws or _default_ws).get(calibrate_absmax_workspace_bytes(rows, cols, gran))
    _check(lib().mpq_calibrate_absmax(_ptr(x), rows, cols, gran, int(accumulate), _ptr(out), wp, wn,
                                      _stream()), "mpq_calibrate_absmax")
    return out


def scale_from_absmax(absmax, bits, out=None):
    torch = _torch()
    if out is None:
        out = torch.empty_like(absmax)
    _check(lib().mpq_scale_from_absmax(_ptr(absmax), absmax.numel(), bits, _ptr(out), _stream()),
           "mpq_scale_from_absmax")
    return out


def fake_quant(x, absmax, bits, gran=PER_TENSOR, want_y=True, want_codes=False, want_packed4=False,
               y=None, codes=None, packed4=None):
    """Returns (y | None, codes | None, packed4 | None)."""
    torch = _torch()
    x = _dev2d(x, torch.float32)
    rows, cols = x.shape
    if want_y and y is None:
        y = torch.empty_like(x)
    if want_codes and codes is None:
        codes = torch.empty((rows, cols), dtype=torch.int8, device=x.device)
    if want_packed4 and packed4 is None:
        packed4 = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
    _check(lib().mpq_fake_quant(_ptr(x), rows, cols, gran, _ptr(absmax), bits, _ptr(y), _ptr(codes),
                                _ptr(packed4), _stream()), "mpq_fake_quant")
    return y, codes, packed4


def fake_quant_step(x, absmax, bits, want_y=True, want_codes=False, want_packed4=False, y=None, codes=None,
                    packed4=None, step=None):
    """Per-tensor fake_quant whose kernel also leaves the step size absmax / qmax_b.
    Returns (y | None, codes | None, packed4 | None, step float32[1])."""
    torch = _torch()
    x = _dev2d(x, torch.float32)
    rows, cols = x.shape
    if want_y and y is None:
        y = torch.empty_like(x)
    if want_codes and codes is None:
        codes = torch.empty((rows, cols), dtype=torch.int8, device=x.device)
    if want_packed4 and packed4 is None:
        packed4 = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
    if step is None:
        step = torch.empty(1, dtype=torch.float32, device=x.device)
    _check(lib().mpq_fake_quant_step(_ptr(x), rows, cols, _ptr(absmax), bits, _ptr(y), _ptr(codes), _ptr(packed4),
                                     _ptr(step), _stream()), "mpq_fake_quant_step")
    return y, codes, packed4, step


def quant_error_workspace_bytes(rows, cols, gran=PER_TENSOR, b_lo=2, b_hi=8) -> int:
    return int(lib().mpq_quant_error_workspace_bytes(rows, cols, gran, b_lo, b_hi))


def quant_error(x, absmax, b_lo=2, b_hi=8, gran=PER_TENSOR, out=None, ws: Workspace = None):
    """Returns float64 [nch, nb] on the device."""
    torch = _torch()
    x = _dev2d(x, torch.float32)
    rows, cols = x.shape
    nb = b_hi - b_lo + 1
    if out is None:
        out = torch.empty((_nch(gran, rows, cols), max(nb, 1)), dtype=torch.float64, device=x.device)
    wp, wn = (ws or _default_ws).get(quant_error_workspace_bytes(rows, cols, gran, b_lo, b_hi))
    _check(lib().mpq_quant_error(_ptr(x), rows, cols, gran, _ptr(absmax), b_lo, b_hi, _ptr(out), wp,
                                 wn, _stream()), "mpq_quant_error")
    return out


def quant_error_noalloc(x, absmax, out, b_lo=2, b_hi=8, gran=PER_TENSOR):
    """quant_error without a workspace and without any allocation, here or in the library: the
    caller passes the float64 [nch, nb] output; partial sums go to the library's built-in buffer."""
    rows, cols = x.shape
    _check(lib().mpq_quant_error_noalloc(_ptr(x), rows, cols, gran, _ptr(absmax), b_lo, b_hi, _ptr(out),
                                         _stream()), "mpq_quant_error_noalloc")
    return out


SWEEP_TENSOR_AND_ROW = 3


def eqe(sse: float, n: int, absmax: float) -> float:
    """Eq. 2 from an error sum read back from the device (host arithmetic in the library)."""
    return float(lib().mpq_eqe(float(sse), int(n), float(absmax)))


def eqe_channels(sse_ch, n: int, absmax_ch):
    """Eq. 2 of a tensor with one scale per channel, from host arrays sse_ch [nch, nb] (float64) and
    absmax_ch [nch] (float32); returns a list of nb values."""
    import numpy as np
    s = np.ascontiguousarray(sse_ch, dtype=np.float64)
    m = np.ascontiguousarray(absmax_ch, dtype=np.float32).ravel()
    if s.ndim != 2 or s.shape[0] != m.size:
        raise ValueError("sse_ch must be [nch, nb] with one absmax per channel")
    out = (C.c_double * s.shape[1])()
    _check(lib().mpq_eqe_channels(s.ctypes.data, m.ctypes.data, m.size, s.shape[1], int(n), out), "mpq_eqe_channels")
    return list(out)


def latency_estimate(layer_us, width_index) -> float:
    """Model latency of a configuration: layer_us [n_layers, n_widths] measured kernel latencies,
    width_index[l] the candidate precision number of layer l (host arithmetic in the library)."""
    import numpy as np
    t = np.ascontiguousarray(layer_us, dtype=np.float64)
    if t.ndim != 2 or t.shape[0] != len(width_index):
        raise ValueError("one row of kernel latencies and one width index per layer")
    idx = (C.c_int * t.shape[0])(*[int(v) for v in width_index])
    out = C.c_double(0.0)
    _check(lib().mpq_latency_estimate(t.ctypes.data, t.shape[0], t.shape[1], idx, C.byref(out)), "mpq_latency_estimate")
    return out.value


def model_size_bytes(parameters, bits) -> float:
    """Parameters times their bit-widths, in bytes (host arithmetic in the library)."""
    n = len(parameters)
    if n != len(bits):
        raise ValueError("one bit-width per layer")
    p = (C.c_int64 * n)(*[int(v) for v in parameters])
    b = (C.c_int * n)(*[int(v) for v in bits])
    out = C.c_double(0.0)
    _check(lib().mpq_model_size_bytes(p, b, n, C.byref(out)), "mpq_model_size_bytes")
    return out.value


def hutchinson_trace(quad, rows: int):
    """(estimate, standard error) of the Hessian trace from the quadratic forms read back from the
    device (host array of P float64) of a tensor with `rows` rows."""
    import numpy as np
    q = np.ascontiguousarray(quad, dtype=np.float64).ravel()
    est, err = C.c_double(0.0), C.c_double(0.0)
    _check(lib().mpq_hutchinson_trace(q.ctypes.data, q.size, int(rows), C.byref(est), C.byref(err)), "mpq_hutchinson_trace")
    return est.value, err.value


class SweepTensor(C.Structure):
    """mpq_sweep_tensor of include/mpq.h: a host struct of device pointers."""
    _fields_ = [("x", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64), ("absmax_row", C.c_void_p),
                ("absmax_tensor", C.c_void_p), ("sse_tensor", C.c_void_p), ("sse_row", C.c_void_p)]


class SweepPlan:
    """The plan of the batched sweep calls for a fixed set of 2-D fp32 device tensors: allocates
    the result buffers (absmax_row / absmax_tensor / sse_tensor / sse_row per tensor), has the
    library build the plan in host memory and uploads the bytes.  Keeps everything alive."""

    def __init__(self, tensors, b_lo=2, b_hi=8):
        torch = _torch()
        self.tensors = [_dev2d(t, torch.float32) for t in tensors]
        self.b_lo, self.b_hi = b_lo, b_hi
        nb = b_hi - b_lo + 1
        dev = self.tensors[0].device
        f32, f64 = torch.float32, torch.float64
        n = len(self.tensors)
        rows = [t.shape[0] for t in self.tensors]
        # one buffer per kind, cut into per-tensor views: results of a sweep read back in one copy
        self.absmax_row_all = torch.empty(sum(rows), dtype=f32, device=dev)
        self.absmax_tensor_all = torch.empty(n, dtype=f32, device=dev)
        self.sse_tensor_all = torch.empty((n, nb), dtype=f64, device=dev)
        self.sse_row_all = torch.empty((sum(rows), nb), dtype=f64, device=dev)
        self.absmax_row, self.absmax_tensor, self.sse_tensor, self.sse_row = [], [], [], []
        r0 = 0
        for i, r in enumerate(rows):
            self.absmax_row.append(self.absmax_row_all[r0:r0 + r])
            self.absmax_tensor.append(self.absmax_tensor_all[i:i + 1])
            self.sse_tensor.append(self.sse_tensor_all[i:i + 1])
            self.sse_row.append(self.sse_row_all[r0:r0 + r])
            r0 += r
        self.desc = (SweepTensor * n)()
        for i, t in enumerate(self.tensors):
            self.desc[i] = SweepTensor(t.data_ptr(), t.shape[0], t.shape[1], self.absmax_row[i].data_ptr(),
                                       self.absmax_tensor[i].data_ptr(), self.sse_tensor[i].data_ptr(),
                                       self.sse_row[i].data_ptr())
        nbytes = int(lib().mpq_sweep_plan_bytes(self.desc, n))
        self.host = (C.c_uint64 * ((max(nbytes, 8) + 7) // 8))()
        _check(lib().mpq_sweep_plan_build(self.desc, n, self.host, C.sizeof(self.host)), "mpq_sweep_plan_build")
        self.nbytes = nbytes
        self.dev = torch.frombuffer(self.host, dtype=torch.uint8).cuda()   # the caller uploads the plan
        self.ws = Workspace()


def sweep_plan_bytes(plan: "SweepPlan") -> int:
    return plan.nbytes


def sweep_plan_build(tensors, b_lo=2, b_hi=8) -> "SweepPlan":
    return SweepPlan(tensors, b_lo, b_hi)


def calibrate_absmax_batch(plan: "SweepPlan"):
    """Row maxima and tensor maxima of every tensor of the plan; results in plan.absmax_row / absmax_tensor."""
    _check(lib().mpq_calibrate_absmax_batch(plan.host, plan.dev.data_ptr(), _stream()), "mpq_calibrate_absmax_batch")
    return plan


def calibrate_quant_error_rows_batch(plan: "SweepPlan"):
    """Row and tensor maxima AND the per-row error sums of every tensor of the plan from one read."""
    _check(lib().mpq_calibrate_quant_error_rows_batch(plan.host, plan.dev.data_ptr(), plan.b_lo, plan.b_hi, _stream()),
           "mpq_calibrate_quant_error_rows_batch")
    return plan


def quant_error_batch_workspace_bytes(plan: "SweepPlan", gran=PER_TENSOR) -> int:
    return int(lib().mpq_quant_error_batch_workspace_bytes(plan.host, gran, plan.b_lo, plan.b_hi))


def quant_error_batch(plan: "SweepPlan", gran=PER_TENSOR):
    """Eq. 2's sums of every tensor of the plan (results in plan.sse_tensor / plan.sse_row)."""
    wp, wn = plan.ws.get(quant_error_batch_workspace_bytes(plan, gran))
    _check(lib().mpq_quant_error_batch(plan.host, plan.dev.data_ptr(), gran, plan.b_lo, plan.b_hi, wp, wn, _stream()),
           "mpq_quant_error_batch")
    return plan


def noise_inject(x, absmax, bits, lam, seed, stream_id, gran=PER_TENSOR, out=None):
    torch = _torch()
    x = _dev2d(x, torch.float32)
    rows, cols = x.shape
    if out is None:
        out = torch.empty_like(x)
    _check(lib().mpq_noise_inject(_ptr(x), rows, cols, gran, _ptr(absmax), bits, float(lam),
                                  int(seed), int(stream_id), _ptr(out), _stream()), "mpq_noise_inject")
    return out


def noise_inject_sweep(x, absmax, b_lo, b_hi, lam, seed, stream_id, gran=PER_TENSOR, out=None):
    """Noise at every bit-width b_lo..b_hi in one pass; returns fp32 [nb, rows, cols]."""
    torch = _torch()
    x = _dev2d(x, torch.float32)
    rows, cols = x.shape
    nb = b_hi - b_lo + 1
    if out is None:
        out = torch.empty((max(nb, 1), rows, cols), dtype=torch.float32, device=x.device)
    if out.dim() != 3 or tuple(out.shape[1:]) != (rows, cols) or not out[0].is_contiguous():
        raise ValueError("noise_inject_sweep needs an output of shape [nb, rows, cols] with contiguous planes")
    _check(lib().mpq_noise_inject_sweep(_ptr(x), rows, cols, gran, _ptr(absmax), b_lo, b_hi, float(lam), int(seed),
                                        int(stream_id), _ptr(out), out.stride(0), _stream()), "mpq_noise_inject_sweep")
    return out


def qgemm_workspace_bytes(M, N, K, w_storage_bits=8) -> int:
    return int(lib().mpq_qgemm_workspace_bytes(M, N, K, w_storage_bits))


def qgemm(a_q, w_q, a_scale, w_scale, w_storage_bits=8, w_gran=PER_TENSOR, want_y=True,
          want_acc=False, y=None, acc=None, ws: Workspace = None, use_workspace=True):
    """Returns (Y fp32 [M,N] | None, acc int32 [M,N] | None).  use_workspace=False passes no
    workspace: shapes the library would cut along K are then computed unsplit (same results)."""
    torch = _torch()
    a_q = _dev2d(a_q, torch.int8)
    M, K = a_q.shape
    N = w_q.shape[0]
    if want_y and y is None:
        y = torch.empty((M, N), dtype=torch.float32, device=a_q.device)
    if want_acc and acc is None:
        acc = torch.empty((M, N), dtype=torch.int32, device=a_q.device)
    wp, wn = (ws or _default_ws).get(qgemm_workspace_bytes(M, N, K, w_storage_bits)) if use_workspace else (None, 0)
    _check(lib().mpq_qgemm(_ptr(a_q), _ptr(w_q), w_storage_bits, M, N, K, _ptr(a_scale),
                           _ptr(w_scale), w_gran, _ptr(y), _ptr(acc), wp, wn, _stream()), "mpq_qgemm")
    return y, acc


def sse_pair_workspace_bytes(n) -> int:
    return int(lib().mpq_sse_pair_workspace_bytes(n))


def sse_pair(y, y_ref, out=None, ws: Workspace = None):
    torch = _torch()
    n = y.numel()
    if y_ref.numel() != n or y.dtype != torch.float32 or y_ref.dtype != torch.float32:
        raise ValueError("sse_pair needs two fp32 tensors of equal size")
    if not (y.is_contiguous() and y_ref.is_contiguous()):
        raise ValueError("sse_pair needs contiguous tensors")
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=y.device)
    wp, wn = (ws or _default_ws).get(sse_pair_workspace_bytes(n))
    _check(lib().mpq_sse_pair(_ptr(y), _ptr(y_ref), n, _ptr(out), wp, wn, _stream()), "mpq_sse_pair")
    return out


def rademacher(seed: int, stream_id: int, rows: int, cols: int, out=None, device=None):
    """Random signs (+1 / -1, fp32 [rows x cols]) for Hutchinson's estimator, one Philox bit each."""
    torch = _torch()
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.float32, device=device or torch.device("cuda", torch.cuda.current_device()))
    elif out.dtype != torch.float32 or not out.is_contiguous() or out.numel() != rows * cols:
        raise ValueError("rademacher needs a contiguous fp32 output of rows * cols elements")
    _check(lib().mpq_rademacher(seed & (2 ** 64 - 1), stream_id & (2 ** 64 - 1), rows, cols, _ptr(out), _stream()),
           "mpq_rademacher")
    return out


class StackLayer(C.Structure):
    """mpq_stack_layer of include/mpq.h: host arrays of device pointers."""
    _fields_ = [("N", C.c_int64), ("K", C.c_int64), ("n_widths", C.c_int),
                ("w_q", C.POINTER(C.c_void_p)), ("w_scale", C.POINTER(C.c_void_p)),
                ("w_storage_bits", C.POINTER(C.c_int)), ("a_codes", C.c_void_p), ("h", C.c_void_p)]


class StackPlan:
    """The argument block of mpq_stack_evaluate for a fixed stack, built once: per layer the weight
    codes / step sizes / storage widths of every candidate width, the code buffer of its input and
    its fp32 output.  Keeps the tensors alive."""

    def __init__(self, M, layers, a_absmax, a_scale, y_ref, act_bits, act, w_gran):
        """layers: list of dicts {N, K, w_q: [tensor], w_scale: [tensor], store: [int], a_codes: tensor,
        h: tensor | None} in stack order."""
        self.keep = (layers, a_absmax, a_scale, y_ref)
        n = len(layers)
        self.arr = (StackLayer * n)()
        self._hold = []
        for i, L in enumerate(layers):
            nw = len(L["w_q"])
            wq = (C.c_void_p * nw)(*[t.data_ptr() for t in L["w_q"]])
            ws_ = (C.c_void_p * nw)(*[t.data_ptr() for t in L["w_scale"]])
            st = (C.c_int * nw)(*[int(b) for b in L["store"]])
            self._hold += [wq, ws_, st]
            self.arr[i] = StackLayer(L["N"], L["K"], nw, C.cast(wq, C.POINTER(C.c_void_p)),
                                     C.cast(ws_, C.POINTER(C.c_void_p)), C.cast(st, C.POINTER(C.c_int)),
                                     L["a_codes"].data_ptr(), None if L["h"] is None else L["h"].data_ptr())
        self.n, self.M = n, int(M)
        self.a_absmax, self.a_scale, self.y_ref = a_absmax, a_scale, y_ref
        self.act_bits, self.act, self.w_gran = int(act_bits), int(act), int(w_gran)
        self.idx = (C.c_int * n)()
        self.ws_bytes = int(lib().mpq_stack_evaluate_workspace_bytes(self.arr, n, self.M))

    def evaluate(self, width_index, sse_out, ws: "Workspace" = None):
        """Enqueues one evaluation with layer l at its candidate width number width_index[l]."""
        for i, w in enumerate(width_index):
            self.idx[i] = int(w)
        wp, wn = (ws or _default_ws).get(self.ws_bytes)
        _check(lib().mpq_stack_evaluate(self.arr, self.n, self.M, self.idx, self.act_bits, self.act, self.w_gran,
                                        _ptr(self.a_absmax), _ptr(self.a_scale), _ptr(self.y_ref), _ptr(sse_out),
                                        wp, wn, _stream()), "mpq_stack_evaluate")
        return sse_out


def stack_evaluate_workspace_bytes(plan: "StackPlan") -> int:
    return plan.ws_bytes


def stack_evaluate(plan: "StackPlan", width_index, sse_out, ws: "Workspace" = None):
    """One evaluation of a stack (see StackPlan): layer l at its candidate width number width_index[l]."""
    return plan.evaluate(width_index, sse_out, ws)


def diag_mfma_operand_bytes() -> int:
    return int(lib().mpq_diag_mfma_operand_bytes())


def diag_mfma_rate(operands, iters: int = 2048, reps: int = 5) -> float:
    """Measured int8 matrix-core issue rate in TOP/s for operand registers filled from `operands`
    (device int8 tensor of at least diag_mfma_operand_bytes() bytes): a measurement aid."""
    torch = _torch()
    sink = torch.zeros(1, dtype=torch.int32, device=operands.device)
    ops = C.c_double(0.0)
    nbytes = operands.numel() * operands.element_size()

    def launch():
        _check(lib().mpq_diag_mfma_rate(_ptr(operands), nbytes, iters, _ptr(sink), C.byref(ops), _stream()),
               "mpq_diag_mfma_rate")

    launch()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        launch()
    e1.record()
    torch.cuda.synchronize()
    return ops.value * reps / (e0.elapsed_time(e1) * 1e-3) / 1e12


def diag_sweep_alu_rate(iters: int = 1000, reps: int = 5) -> float:
    """Measured rate, in T lane-operations per second, of the error sweep's arithmetic (b = 2..8, 28
    lane-operations per element) on elements held in registers: a measurement aid."""
    torch = _torch()
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    ops = C.c_double(0.0)

    def launch():
        _check(lib().mpq_diag_sweep_alu_rate(iters, _ptr(sink), C.byref(ops), _stream()), "mpq_diag_sweep_alu_rate")

    launch()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        launch()
    e1.record()
    torch.cuda.synchronize()
    return ops.value * reps / (e0.elapsed_time(e1) * 1e-3) / 1e12


def hutchinson_quad_workspace_bytes(M, K, P) -> int:
    return int(lib().mpq_hutchinson_quad_workspace_bytes(M, K, P))


def hutchinson_quad(x, v, out=None, ws: Workspace = None):
    """quad[p] = ||X v_p||^2 for the rows v_p of v (float64 [P]): the quadratic forms of Hutchinson's
    trace estimate for a linear layer under a mean-squared-error loss."""
    torch = _torch()
    x, v = _dev2d(x, torch.float32), _dev2d(v, torch.float32)
    M, K = x.shape
    P = v.shape[0]
    if v.shape[1] != K:
        raise ValueError("probes need as many columns as x")
    if out is None:
        out = torch.empty(P, dtype=torch.float64, device=x.device)
    wp, wn = (ws or _default_ws).get(hutchinson_quad_workspace_bytes(M, K, P))
    _check(lib().mpq_hutchinson_quad(_ptr(x), M, K, _ptr(v), P, _ptr(out), wp, wn, _stream()), "mpq_hutchinson_quad")
    return out


def hutchinson_quad_signs(x, seed: int, stream_id: int, probes: int, out=None, ws: Workspace = None):
    """hutchinson_quad for the sign probes rademacher(seed, stream_id, probes, K) would store, drawn
    inside the kernel (K % 16 == 0, x 16-byte aligned)."""
    torch = _torch()
    x = _dev2d(x, torch.float32)
    M, K = x.shape
    if out is None:
        out = torch.empty(probes, dtype=torch.float64, device=x.device)
    wp, wn = (ws or _default_ws).get(hutchinson_quad_workspace_bytes(M, K, probes))
    _check(lib().mpq_hutchinson_quad_signs(_ptr(x), M, K, seed & (2 ** 64 - 1), stream_id & (2 ** 64 - 1), probes,
                                           _ptr(out), wp, wn, _stream()), "mpq_hutchinson_quad_signs")
    return out


def qgemm_score_workspace_bytes(M, N, K, w_storage_bits=8) -> int:
    return int(lib().mpq_qgemm_score_workspace_bytes(M, N, K, w_storage_bits))


def qgemm_score(a_q, w_q, a_scale, w_scale, y_ref, w_storage_bits=8, w_gran=PER_TENSOR, want_y=False,
                y=None, out=None, ws: Workspace = None):
    """One quantized layer scored against y_ref in its epilogue.  Returns (sse float64[1], Y | None)."""
    torch = _torch()
    a_q = _dev2d(a_q, torch.int8)
    M, K = a_q.shape
    N = w_q.shape[0]
    if y_ref.dtype != torch.float32 or tuple(y_ref.shape) != (M, N) or not y_ref.is_contiguous():
        raise ValueError("qgemm_score needs a contiguous fp32 y_ref of shape [M, N]")
    if want_y and y is None:
        y = torch.empty((M, N), dtype=torch.float32, device=a_q.device)
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=a_q.device)
    wp, wn = (ws or _default_ws).get(qgemm_score_workspace_bytes(M, N, K, w_storage_bits))
    _check(lib().mpq_qgemm_score(_ptr(a_q), _ptr(w_q), w_storage_bits, M, N, K, _ptr(a_scale), _ptr(w_scale),
                                 w_gran, _ptr(y_ref), _ptr(out), _ptr(y), wp, wn, _stream()), "mpq_qgemm_score")
    return out, y


def _search(fn, name, order, bit_widths, target, evaluate, flags):
    n, nb = len(order), len(bit_widths)
    c_order = (C.c_int * n)(*[int(v) for v in order])
    c_bits = (C.c_int * nb)(*[int(v) for v in bit_widths])
    out = (C.c_int * max(n, 1))()
    n_evals = C.c_int(0)
    failure = []

    def trampoline(bits, n_layers, _user):
        if failure:                       # an earlier evaluation raised: let the search run out
            return float("-inf")
        try:
            return float(evaluate([bits[i] for i in range(n_layers)]))
        except BaseException as e:        # never unwind through the C frames
            failure.append(e)
            return float("-inf")

    cb = EVAL_FN(trampoline)
    _check(fn(c_order, n, c_bits, nb, float(target), int(flags), cb, None, out, C.byref(n_evals)), name)
    if failure:
        raise failure[0]
    return [out[i] for i in range(n)], n_evals.value


def search_bisection(order, bit_widths, target, evaluate, ensure_target=False):
    """Alg. 1.  order: layer ids by ascending sensitivity; evaluate(bits per layer) -> accuracy.
    Returns (bits per layer, number of evaluations)."""
    return _search(lib().mpq_search_bisection, "mpq_search_bisection", order, bit_widths, target, evaluate,
                   SEARCH_ENSURE_TARGET if ensure_target else 0)


def search_greedy(order, bit_widths, target, evaluate):
    """Alg. 2.  Same arguments and result as search_bisection."""
    return _search(lib().mpq_search_greedy, "mpq_search_greedy", order, bit_widths, target, evaluate, 0)


def fake_quant_scales(x, inv, scale, bits, gran=PER_TENSOR, want_y=True, want_codes=False):
    """Eq. 1 with explicit scales (after adjustment they no longer derive from one absmax)."""
    torch = _torch()
    x = _dev2d(x, torch.float32)
    rows, cols = x.shape
    y = torch.empty_like(x) if want_y else None
    codes = torch.empty((rows, cols), dtype=torch.int8, device=x.device) if want_codes else None
    _check(lib().mpq_fake_quant_scales(_ptr(x), rows, cols, gran, _ptr(inv), _ptr(scale), bits, _ptr(y), _ptr(codes),
                                       _stream()), "mpq_fake_quant_scales")
    return y, codes


def scale_grad_workspace_bytes(rows, cols, gran=PER_TENSOR) -> int:
    return int(lib().mpq_scale_grad_workspace_bytes(rows, cols, gran))


def scale_grad(x, inv, scale, bits, g=None, gran=PER_TENSOR, ws: Workspace = None):
    """Straight-through gradients of the two scales.  Returns (dinv, dscale, loss), float64 [nch]."""
    torch = _torch()
    x = _dev2d(x, torch.float32)
    rows, cols = x.shape
    nch = _nch(gran, rows, cols)
    if g is not None:
        g = _dev2d(g, torch.float32)
        if g.shape != x.shape:
            raise ValueError("the upstream gradient must have the tensor's shape")
    out = [torch.empty(nch, dtype=torch.float64, device=x.device) for _ in range(3)]
    wp, wn = (ws or _default_ws).get(scale_grad_workspace_bytes(rows, cols, gran))
    _check(lib().mpq_scale_grad(_ptr(x), rows, cols, gran, _ptr(inv), _ptr(scale), bits, _ptr(g), _ptr(out[0]),
                                _ptr(out[1]), _ptr(out[2]), wp, wn, _stream()), "mpq_scale_grad")
    return tuple(out)


def scale_sgd_step(inv, scale, dinv, dscale, lr):
    """In place: inv -= lr * dinv, scale -= lr * dscale (double arithmetic, one rounding)."""
    n = inv.numel()
    if not (scale.numel() == dinv.numel() == dscale.numel() == n):
        raise ValueError("scale vectors and gradients must have one entry per channel")
    _check(lib().mpq_scale_sgd_step(_ptr(inv), _ptr(scale), _ptr(dinv), _ptr(dscale), n, float(lr), _stream()),
           "mpq_scale_sgd_step")
    return inv, scale


def qgemm_act(a_q, w_q, a_scale, w_scale, act, w_storage_bits=8, w_gran=PER_TENSOR, y=None, absmax=None,
              want_absmax=True, accumulate=False, want_y=True):
    """One quantized layer with its activation (ACT_RELU / ACT_GELU) applied in the epilogue and,
    if wanted, the absmax of the activated output.  Returns (Y | None, absmax float32[1] | None);
    want_y=False is the calibration-only pass that stores no layer output."""
    torch = _torch()
    a_q = _dev2d(a_q, torch.int8)
    M, K = a_q.shape
    N = w_q.shape[0]
    if y is None and want_y:
        y = torch.empty((M, N), dtype=torch.float32, device=a_q.device)
    if want_absmax and absmax is None:
        if accumulate:
            raise ValueError("a running maximum needs the caller's absmax tensor")
        absmax = torch.empty(1, dtype=torch.float32, device=a_q.device)
    _check(lib().mpq_qgemm_act(_ptr(a_q), _ptr(w_q), w_storage_bits, M, N, K, _ptr(a_scale), _ptr(w_scale), w_gran,
                               int(act), _ptr(y), _ptr(absmax), 1 if accumulate else 0, _stream()), "mpq_qgemm_act")
    return y, absmax


def qgemm_act_codes(a_q, w_q, a_scale, w_scale, act, absmax, bits, w_storage_bits=8, w_gran=PER_TENSOR, codes=None):
    """The layer of qgemm_act with its activated output quantized in the epilogue (Eq. 1 with the
    given absmax): returns the int8 codes [M x N]; the fp32 output is never stored."""
    torch = _torch()
    a_q = _dev2d(a_q, torch.int8)
    M, K = a_q.shape
    N = w_q.shape[0]
    if codes is None:
        codes = torch.empty((M, N), dtype=torch.int8, device=a_q.device)
    _check(lib().mpq_qgemm_act_codes(_ptr(a_q), _ptr(w_q), w_storage_bits, M, N, K, _ptr(a_scale), _ptr(w_scale),
                                     w_gran, int(act), _ptr(absmax), int(bits), _ptr(codes), _stream()),
           "mpq_qgemm_act_codes")
    return codes
