"""ctypes front end of the CPU oracle (``mpq_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
cpu_baseline leg.  The product package never imports this module.

The shared object is rebuilt with g++ whenever the source is newer than it; the oracle has no
dependency besides libstdc++/libm.  Arrays are numpy arrays; shapes are 2-D row-major.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mpq_oracle.cpp")
_LIB = os.path.join(_HERE, "libmpq_oracle.so")

PER_TENSOR, PER_ROW, PER_COL = 0, 1, 2
OK, BAD_ARG, ACC_OVERFLOW = 0, 1, 2

# no -march flags, contraction off: every fp32 step in the source is exactly one IEEE operation
CXXFLAGS = ["-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]


# MPQ_ORACLE_SANITIZE=1 builds (and loads) a second copy of the oracle instrumented with the address and
# undefined-behaviour sanitizers.  Python itself is not instrumented, so the sanitizer runtime has
# to be in the process first:
#   LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 MPQ_ORACLE_SANITIZE=1 \
#       python -m pytest tests -m "not gpu"
SANITIZE = os.environ.get("MPQ_ORACLE_SANITIZE", "0") not in ("", "0")
_SAN_LIB = os.path.join(_HERE, "libmpq_oracle_san.so")
SAN_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]


def build(force: bool = False) -> str:
    out = _SAN_LIB if SANITIZE else _LIB
    stale = (not os.path.exists(out)) or os.path.getmtime(out) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = out + ".tmp%d" % os.getpid()
        subprocess.check_call(["g++", *CXXFLAGS, *(SAN_FLAGS if SANITIZE else []), "-o", tmp, _SRC])
        os.replace(tmp, out)
    return out


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_eqe.restype = C.c_double
        _lib.orc_sse_pair.restype = C.c_double
        _lib.orc_neg2log_u24.restype = C.c_float
        _lib.orc_neg2log_u24.argtypes = [C.c_uint32]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32_2d(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim != 2:
        raise ValueError("oracle tensors are 2-D [rows x cols]")
    return x


def _nch(gran, rows, cols):
    return {PER_TENSOR: 1, PER_ROW: rows, PER_COL: cols}[gran]


def _check(rc, what):
    if rc != OK:
        raise RuntimeError("oracle %s failed with code %d" % (what, rc))


def qmax(bits: int) -> int:
    return int(lib().orc_qmax(C.c_int(bits)))


def absmax(x, gran=PER_TENSOR, running=None):
    """Sec. 3.1 calibration maximum.  ``running``: previous result to keep a running maximum."""
    x = _f32_2d(x)
    rows, cols = x.shape
    out = np.zeros(_nch(gran, rows, cols), dtype=np.float32)
    acc = 0
    if running is not None:
        out[:] = np.asarray(running, dtype=np.float32)
        acc = 1
    _check(lib().orc_absmax(_p(x), C.c_int64(rows), C.c_int64(cols), C.c_int(gran), C.c_int(acc),
                            _p(out)), "absmax")
    return out


def bit_constants(m: float, bits: int):
    s, i = C.c_float(), C.c_float()
    lib().orc_bit_constants(C.c_float(m), C.c_int(bits), C.byref(s), C.byref(i))
    return np.float32(s.value), np.float32(i.value)


def scale_from_absmax(absmax_arr, bits: int):
    a = np.ascontiguousarray(absmax_arr, dtype=np.float32).ravel()
    out = np.empty_like(a)
    lib().orc_scale_from_absmax(_p(a), C.c_int64(a.size), C.c_int(bits), _p(out))
    return out


def fake_quant(x, absmax_arr, bits, gran=PER_TENSOR, want_packed4=False):
    """Eq. 1.  Returns (y fp32, codes int8, packed4 uint8 | None)."""
    x = _f32_2d(x)
    rows, cols = x.shape
    am = np.ascontiguousarray(absmax_arr, dtype=np.float32).ravel()
    assert am.size == _nch(gran, rows, cols)
    y = np.empty_like(x)
    codes = np.empty(x.shape, dtype=np.int8)
    packed = np.zeros((rows, cols // 2), dtype=np.uint8) if want_packed4 else None
    _check(lib().orc_fake_quant(_p(x), C.c_int64(rows), C.c_int64(cols), C.c_int(gran), _p(am),
                                C.c_int(bits), _p(y), _p(codes), _p(packed)), "fake_quant")
    return y, codes, packed


def quant_error(x, absmax_arr, b_lo=2, b_hi=8, gran=PER_TENSOR):
    """Eq. 2 sums.  Returns float64 [nch, nb]."""
    x = _f32_2d(x)
    rows, cols = x.shape
    am = np.ascontiguousarray(absmax_arr, dtype=np.float32).ravel()
    nch = _nch(gran, rows, cols)
    assert am.size == nch
    out = np.empty((nch, b_hi - b_lo + 1), dtype=np.float64)
    _check(lib().orc_quant_error(_p(x), C.c_int64(rows), C.c_int64(cols), C.c_int(gran), _p(am),
                                 C.c_int(b_lo), C.c_int(b_hi), _p(out)), "quant_error")
    return out


def eqe(sse: float, n: int, m: float) -> float:
    return float(lib().orc_eqe(C.c_double(sse), C.c_int64(n), C.c_float(m)))


def eqe_channels(sse_ch, n: int, absmax_ch):
    """Eq. 2 of a tensor quantized with one scale per channel, from its channels' error sums
    [nch, nb] and maxima [nch]: float64 [nb]."""
    s = np.ascontiguousarray(sse_ch, dtype=np.float64)
    m = np.ascontiguousarray(absmax_ch, dtype=np.float32).ravel()
    assert s.ndim == 2 and s.shape[0] == m.size
    out = np.empty(s.shape[1], np.float64)
    lib().orc_eqe_channels(_p(s), _p(m), C.c_int64(m.size), C.c_int(s.shape[1]), C.c_int64(n), _p(out))
    return out


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (C.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(v) for v in o]


def neg2log_u24(k: int) -> np.float32:
    return np.float32(lib().orc_neg2log_u24(C.c_uint32(k)))


def sincos_2pi_u24(j: int):
    c, s = C.c_float(), C.c_float()
    lib().orc_sincos_2pi_u24(C.c_uint32(j), C.byref(c), C.byref(s))
    return np.float32(c.value), np.float32(s.value)


def gauss4(seed: int, stream_id: int, g: int):
    z = (C.c_float * 4)()
    lib().orc_gauss4(C.c_uint64(seed), C.c_uint64(stream_id), C.c_uint64(g), z)
    return np.array(list(z), dtype=np.float32)


def noise_inject(x, absmax_arr, bits, lam, seed, stream_id, gran=PER_TENSOR):
    """Eq. 3-5: x + sigma z."""
    x = _f32_2d(x)
    rows, cols = x.shape
    am = np.ascontiguousarray(absmax_arr, dtype=np.float32).ravel()
    assert am.size == _nch(gran, rows, cols)
    y = np.empty_like(x)
    _check(lib().orc_noise_inject(_p(x), C.c_int64(rows), C.c_int64(cols), C.c_int(gran), _p(am),
                                  C.c_int(bits), C.c_float(lam), C.c_uint64(seed),
                                  C.c_uint64(stream_id), _p(y)), "noise_inject")
    return y


def noise_inject_sweep(x, absmax_arr, b_lo, b_hi, lam, seed, stream_id, gran=PER_TENSOR):
    """Eq. 3-5 at every bit-width b_lo..b_hi: by definition one noise_inject per b (the draw z does not
    depend on b, so all planes share it).  Returns [nb, rows, cols]."""
    return np.stack([noise_inject(x, absmax_arr, b, lam, seed, stream_id, gran) for b in range(b_lo, b_hi + 1)])


def pack4(codes):
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    assert codes.size % 2 == 0
    out = np.empty(codes.size // 2, dtype=np.uint8)
    lib().orc_pack4(_p(codes), C.c_int64(out.size), _p(out))
    return out.reshape(codes.shape[:-1] + (codes.shape[-1] // 2,))


def unpack4(packed):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    out = np.empty(packed.size * 2, dtype=np.int8)
    lib().orc_unpack4(_p(packed), C.c_int64(packed.size), _p(out))
    return out.reshape(packed.shape[:-1] + (packed.shape[-1] * 2,))


def qgemm(a_q, w_q, a_scale, w_scale, w_storage_bits=8, w_gran=PER_TENSOR):
    """Quantized linear layer.  Returns (Y fp32 [M,N], acc int32 [M,N])."""
    a_q = np.ascontiguousarray(a_q, dtype=np.int8)
    M, K = a_q.shape
    if w_storage_bits == 8:
        w_q = np.ascontiguousarray(w_q, dtype=np.int8)
        N = w_q.shape[0]
        assert w_q.shape[1] == K
    else:
        w_q = np.ascontiguousarray(w_q, dtype=np.uint8)
        N = w_q.shape[0]
        assert w_q.shape[1] * 2 == K
    sa = np.ascontiguousarray(a_scale, dtype=np.float32).ravel()
    sw = np.ascontiguousarray(w_scale, dtype=np.float32).ravel()
    assert sa.size == 1 and sw.size == (N if w_gran == PER_ROW else 1)
    y = np.empty((M, N), dtype=np.float32)
    acc = np.empty((M, N), dtype=np.int32)
    _check(lib().orc_qgemm(_p(a_q), _p(w_q), C.c_int(w_storage_bits), C.c_int64(M), C.c_int64(N),
                           C.c_int64(K), _p(sa), _p(sw), C.c_int(w_gran), _p(y), _p(acc)), "qgemm")
    return y, acc


def sse_pair(y, y_ref) -> float:
    y = np.ascontiguousarray(y, dtype=np.float32).ravel()
    r = np.ascontiguousarray(y_ref, dtype=np.float32).ravel()
    assert y.size == r.size
    return float(lib().orc_sse_pair(_p(y), _p(r), C.c_int64(y.size)))


def rademacher(seed: int, stream_id: int, rows: int, cols: int):
    """Random signs for Hutchinson's estimator (Sec. 3.2.3): float32 [rows x cols] of +-1."""
    v = np.empty((rows, cols), np.float32)
    rc = lib().orc_rademacher(C.c_uint64(seed), C.c_uint64(stream_id), C.c_int64(rows), C.c_int64(cols), _p(v))
    assert rc == 0
    return v


def hutchinson_quad(x, v):
    """quad[p] = ||X v_p||^2 for the rows v_p of v: the quadratic forms of Hutchinson's estimator
    for a linear layer under a mean-squared-error loss (Sec. 3.2.3).  float64 [P]."""
    x, v = _f32_2d(x), _f32_2d(v)
    assert x.shape[1] == v.shape[1]
    q = np.empty(v.shape[0], np.float64)
    rc = lib().orc_hutchinson_quad(_p(x), C.c_int64(x.shape[0]), C.c_int64(x.shape[1]), _p(v),
                                   C.c_int64(v.shape[0]), _p(q))
    assert rc == 0
    return q


def hutchinson_trace(x, v):
    """Estimate of Tr(H) of the layer loss with respect to the weights, (2 / M) mean_p ||X v_p||^2,
    and the standard error of that mean."""
    q = hutchinson_quad(x, v)
    m = _f32_2d(x).shape[0]
    est = 2.0 / m * q.mean()
    err = 2.0 / m * q.std(ddof=1) / np.sqrt(q.size) if q.size > 1 else float("nan")
    return float(est), float(err)


def fake_quant_scales(x, inv, scale, bits, gran=PER_TENSOR):
    """Eq. 1 with explicit scales: returns (Q fp32, codes int8)."""
    x = _f32_2d(x)
    rows, cols = x.shape
    inv = np.ascontiguousarray(inv, dtype=np.float32).ravel()
    scale = np.ascontiguousarray(scale, dtype=np.float32).ravel()
    assert inv.size == scale.size == _nch(gran, rows, cols)
    y, codes = np.empty_like(x), np.empty(x.shape, np.int8)
    _check(lib().orc_fake_quant_scales(_p(x), C.c_int64(rows), C.c_int64(cols), C.c_int(gran), _p(inv), _p(scale),
                                       C.c_int(bits), _p(y), _p(codes)), "fake_quant_scales")
    return y, codes


def scale_grad(x, inv, scale, bits, g=None, gran=PER_TENSOR):
    """Straight-through gradients of the two scales: returns dict(dinv, dscale, loss, abs_dinv,
    abs_dscale), each float64 [nch]."""
    x = _f32_2d(x)
    rows, cols = x.shape
    inv = np.ascontiguousarray(inv, dtype=np.float32).ravel()
    scale = np.ascontiguousarray(scale, dtype=np.float32).ravel()
    nch = _nch(gran, rows, cols)
    assert inv.size == scale.size == nch
    gp = None
    if g is not None:
        g = _f32_2d(g)
        assert g.shape == x.shape
        gp = _p(g)
    out = {k: np.empty(nch, np.float64) for k in ("dinv", "dscale", "loss", "abs_dinv", "abs_dscale")}
    _check(lib().orc_scale_grad(_p(x), C.c_int64(rows), C.c_int64(cols), C.c_int(gran), _p(inv), _p(scale),
                                C.c_int(bits), gp, _p(out["dinv"]), _p(out["dscale"]), _p(out["loss"]),
                                _p(out["abs_dinv"]), _p(out["abs_dscale"])), "scale_grad")
    return out


def scale_sgd_step(inv, scale, dinv, dscale, lr):
    """Returns the updated (inv, scale) as new fp32 arrays."""
    inv = np.array(inv, dtype=np.float32).ravel()
    scale = np.array(scale, dtype=np.float32).ravel()
    dinv = np.ascontiguousarray(dinv, dtype=np.float64).ravel()
    dscale = np.ascontiguousarray(dscale, dtype=np.float64).ravel()
    assert inv.size == scale.size == dinv.size == dscale.size
    _check(lib().orc_scale_sgd_step(_p(inv), _p(scale), _p(dinv), _p(dscale), C.c_int64(inv.size), C.c_double(lr)),
           "scale_sgd_step")
    return inv, scale


ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2


def activation(y, act):
    """ReLU or exact-Phi GELU of an fp32 array (a new array)."""
    out = np.array(y, dtype=np.float32, order="C")
    _check(lib().orc_activation(_p(out), C.c_int64(out.size), C.c_int(act)), "activation")
    return out


def qgemm_act(a_q, w_q, a_scale, w_scale, act, w_storage_bits=8, w_gran=PER_TENSOR):
    """The layer followed by its activation, and the absmax of the result: by definition the
    composition of qgemm, activation and absmax.  Returns (y, absmax float32[1])."""
    y, _ = qgemm(a_q, w_q, a_scale, w_scale, w_storage_bits, w_gran)
    y = activation(y, act)
    return y, absmax(y)
