"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

from paper_2302_01382_amd import mpq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = C.c_void_p(0x1000)   # never dereferenced: validation fails first
FAKE16 = C.c_void_p(0x10000)


def _no_gpu() -> bool:
    try:
        import torch
        return not torch.cuda.is_available()
    except Exception:
        return True


# calls with made-up pointers are only ever issued where nothing could be launched
needs_no_gpu = pytest.mark.skipif(not _no_gpu(), reason="fake-pointer validation runs on GPU-less hosts only")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mpq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mpq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 14
    L = mpq.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(mpq.EXPORTS) == names


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 (and as C++) with warnings on."""
    import shutil
    import subprocess
    hdr = os.path.join(ROOT, "include", "mpq.h")
    for cc, std, lang in (("gcc", "-std=c99", "c"), ("g++", "-std=c++17", "c++")):
        if shutil.which(cc) is None:
            pytest.skip("no host compiler")
        r = subprocess.run([cc, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", lang, hdr],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_binding_module_has_the_same_names():
    for n in declared_functions():
        short = n[len("mpq_"):]
        if short in ("strerror", "last_hip_error", "version", "sweep_plan_bytes", "sweep_plan_build"):
            continue
        assert hasattr(mpq, short), short


def test_strerror_and_version():
    L = mpq.lib()
    assert L.mpq_version() >= 100
    seen = set()
    for code in range(0, 9):
        s = L.mpq_strerror(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert "unknown" in L.mpq_strerror(99).decode()


@needs_no_gpu
def test_calibrate_absmax_validation():
    L = mpq.lib()
    f = L.mpq_calibrate_absmax
    q = L.mpq_calibrate_absmax_workspace_bytes
    assert q(1000, 1000, 0) > 0 and q(1000, 1000, 1) == 0 and q(1000, 1000, 2) == 0 and q(0, 4, 0) == 0
    assert f(None, 4, 4, 0, 0, FAKE, FAKE16, 1 << 20, None) == mpq.ERR_NULL
    assert f(FAKE, 4, 4, 0, 0, None, FAKE16, 1 << 20, None) == mpq.ERR_NULL
    assert f(FAKE, 0, 4, 0, 0, FAKE, FAKE16, 1 << 20, None) == mpq.ERR_SHAPE
    assert f(FAKE, 4, -1, 0, 0, FAKE, FAKE16, 1 << 20, None) == mpq.ERR_SHAPE
    assert f(FAKE, 2 ** 40, 2 ** 40, 0, 0, FAKE, FAKE16, 1 << 20, None) == mpq.ERR_SHAPE
    assert f(FAKE, 4, 4, 3, 0, FAKE, FAKE16, 1 << 20, None) == mpq.ERR_GRAN
    assert f(FAKE, 1000, 1000, 0, 0, FAKE, None, 0, None) == mpq.ERR_WORKSPACE
    assert f(FAKE, 1000, 1000, 0, 0, FAKE, FAKE16, q(1000, 1000, 0) - 1, None) == mpq.ERR_WORKSPACE
    assert f(FAKE, 1000, 1000, 0, 0, FAKE, C.c_void_p(0x10004), 1 << 20, None) == mpq.ERR_ALIGN
    assert L.mpq_scale_from_absmax(FAKE, 4, 9, FAKE, None) == mpq.ERR_BITS
    assert L.mpq_scale_from_absmax(FAKE, 0, 8, FAKE, None) == mpq.ERR_SHAPE
    assert L.mpq_scale_from_absmax(None, 4, 8, FAKE, None) == mpq.ERR_NULL


@needs_no_gpu
def test_fake_quant_validation():
    f = mpq.lib().mpq_fake_quant
    assert f(None, 4, 4, 0, FAKE, 4, FAKE, None, None, None) == mpq.ERR_NULL
    assert f(FAKE, 4, 4, 0, None, 4, FAKE, None, None, None) == mpq.ERR_NULL
    assert f(FAKE, 4, 4, 0, FAKE, 4, None, None, None, None) == mpq.ERR_NULL  # no output at all
    assert f(FAKE, 4, 4, 0, FAKE, 1, FAKE, None, None, None) == mpq.ERR_BITS
    assert f(FAKE, 4, 4, 0, FAKE, 9, FAKE, None, None, None) == mpq.ERR_BITS
    assert f(FAKE, 4, 4, 0, FAKE, 5, None, None, FAKE, None) == mpq.ERR_BITS  # packed needs <= 4
    assert f(FAKE, 4, 5, 0, FAKE, 4, None, None, FAKE, None) == mpq.ERR_SHAPE  # odd cols, packed
    assert f(FAKE, 4, 4, 7, FAKE, 4, FAKE, None, None, None) == mpq.ERR_GRAN
    assert f(FAKE, -4, 4, 0, FAKE, 4, FAKE, None, None, None) == mpq.ERR_SHAPE


@needs_no_gpu
def test_diag_mfma_rate_validation():
    L = mpq.lib()
    need = L.mpq_diag_mfma_operand_bytes()
    assert need == 256 * 8 * 64 * 8 * 16
    f = L.mpq_diag_mfma_rate
    assert f(None, need, 16, FAKE, None, None) == mpq.ERR_NULL
    assert f(FAKE16, need, 16, None, None, None) == mpq.ERR_NULL
    assert f(FAKE16, need - 1, 16, FAKE, None, None) == mpq.ERR_WORKSPACE
    assert f(C.c_void_p(0x10008), need, 16, FAKE, None, None) == mpq.ERR_ALIGN
    assert f(FAKE16, need, 0, FAKE, None, None) == mpq.ERR_SHAPE
    g = L.mpq_diag_sweep_alu_rate
    assert g(16, None, None, None) == mpq.ERR_NULL
    assert g(0, FAKE, None, None) == mpq.ERR_SHAPE
    assert g((1 << 20) + 1, FAKE, None, None) == mpq.ERR_SHAPE


@needs_no_gpu
def test_fake_quant_step_validation():
    f = mpq.lib().mpq_fake_quant_step
    assert f(FAKE, 4, 4, FAKE, 8, FAKE, None, None, None, None) == mpq.ERR_NULL           # no step_out
    assert f(FAKE, 4, 4, FAKE, 8, FAKE, None, None, C.c_void_p(0x1002), None) == mpq.ERR_ALIGN
    assert f(None, 4, 4, FAKE, 8, FAKE, None, None, FAKE, None) == mpq.ERR_NULL
    assert f(FAKE, 4, 4, FAKE, 8, None, None, None, FAKE, None) == mpq.ERR_NULL           # no output
    assert f(FAKE, 4, 4, FAKE, 9, FAKE, None, None, FAKE, None) == mpq.ERR_BITS
    assert f(FAKE, 0, 4, FAKE, 8, FAKE, None, None, FAKE, None) == mpq.ERR_SHAPE
    assert f(FAKE, 4, 3, FAKE, 4, None, None, FAKE, FAKE, None) == mpq.ERR_SHAPE          # packed nibbles need even cols


@needs_no_gpu
def test_quant_error_validation_and_workspace_query():
    L = mpq.lib()
    f = L.mpq_quant_error
    q = L.mpq_quant_error_workspace_bytes
    assert q(0, 4, 0, 2, 8) == 0 and q(4, 4, 0, 1, 8) == 0 and q(4, 4, 5, 2, 8) == 0
    need = q(1000, 1000, 0, 2, 8)
    assert need > 0 and need % 8 == 0
    assert q(1000, 1000, 1, 2, 8) == 0                      # one wave covers a row: no scratch
    assert q(4, 100000, 1, 2, 8) == 4 * 7 * 7 * 8           # 7 segments per row
    assert q(1000, 1000, 2, 2, 8) >= 1000 * 7 * 8
    assert f(None, 4, 4, 0, FAKE, 2, 8, FAKE, FAKE16, 1 << 20, None) == mpq.ERR_NULL
    assert f(FAKE, 4, 4, 0, FAKE, 2, 8, None, FAKE16, 1 << 20, None) == mpq.ERR_NULL
    assert f(FAKE, 4, 4, 0, FAKE, 1, 8, FAKE, FAKE16, 1 << 20, None) == mpq.ERR_BITS
    assert f(FAKE, 4, 4, 0, FAKE, 5, 4, FAKE, FAKE16, 1 << 20, None) == mpq.ERR_BITS
    assert f(FAKE, 4, 4, 0, FAKE, 2, 9, FAKE, FAKE16, 1 << 20, None) == mpq.ERR_BITS
    assert f(FAKE, 1000, 1000, 0, FAKE, 2, 8, FAKE, None, 0, None) == mpq.ERR_WORKSPACE
    assert f(FAKE, 1000, 1000, 0, FAKE, 2, 8, FAKE, FAKE16, need - 1, None) == mpq.ERR_WORKSPACE
    assert f(FAKE, 1000, 1000, 0, FAKE, 2, 8, FAKE, C.c_void_p(0x10008), need, None) == mpq.ERR_ALIGN
    assert f(FAKE, 1000, 1000, 0, FAKE, 2, 8, C.c_void_p(0x1004), FAKE16, need, None) == mpq.ERR_ALIGN
    assert f(FAKE, 4, 4, 4, FAKE, 2, 8, FAKE, FAKE16, 1 << 20, None) == mpq.ERR_GRAN


@needs_no_gpu
def test_noise_validation():
    f = mpq.lib().mpq_noise_inject
    assert f(None, 4, 4, 0, FAKE, 4, 0.5, 1, 2, FAKE, None) == mpq.ERR_NULL
    assert f(FAKE, 4, 4, 0, FAKE, 4, 0.5, 1, 2, None, None) == mpq.ERR_NULL
    assert f(FAKE, 4, 4, 0, FAKE, 0, 0.5, 1, 2, FAKE, None) == mpq.ERR_BITS
    assert f(FAKE, 4, 0, 0, FAKE, 4, 0.5, 1, 2, FAKE, None) == mpq.ERR_SHAPE
    assert f(FAKE, 4, 4, -1, FAKE, 4, 0.5, 1, 2, FAKE, None) == mpq.ERR_GRAN


@needs_no_gpu
def test_noise_sweep_validation():
    f = mpq.lib().mpq_noise_inject_sweep
    assert f(None, 4, 4, 0, FAKE, 2, 8, 0.5, 1, 2, FAKE, 16, None) == mpq.ERR_NULL
    assert f(FAKE, 4, 4, 0, FAKE, 2, 8, 0.5, 1, 2, None, 16, None) == mpq.ERR_NULL
    assert f(FAKE, 4, 4, 0, FAKE, 1, 8, 0.5, 1, 2, FAKE, 16, None) == mpq.ERR_BITS
    assert f(FAKE, 4, 4, 0, FAKE, 5, 4, 0.5, 1, 2, FAKE, 16, None) == mpq.ERR_BITS
    assert f(FAKE, 4, 4, 0, FAKE, 2, 8, 0.5, 1, 2, FAKE, 15, None) == mpq.ERR_SHAPE   # planes would overlap
    assert f(FAKE, 4, 4, 3, FAKE, 2, 8, 0.5, 1, 2, FAKE, 16, None) == mpq.ERR_GRAN


@needs_no_gpu
def test_qgemm_validation():
    L = mpq.lib()
    f = L.mpq_qgemm
    assert L.mpq_qgemm_workspace_bytes(128, 128, 128, 8) == 0
    ok_tail = (FAKE, FAKE, 0, FAKE, None, None, 0, None)
    assert f(None, FAKE, 8, 4, 4, 16, *ok_tail) == mpq.ERR_NULL
    assert f(FAKE, None, 8, 4, 4, 16, *ok_tail) == mpq.ERR_NULL
    assert f(FAKE, FAKE, 8, 4, 4, 16, FAKE, FAKE, 0, None, None, None, 0, None) == mpq.ERR_NULL
    assert f(FAKE, FAKE, 8, 4, 4, 16, None, FAKE, 0, FAKE, None, None, 0, None) == mpq.ERR_NULL
    assert f(FAKE, FAKE, 6, 4, 4, 16, *ok_tail) == mpq.ERR_BITS
    assert f(FAKE, FAKE, 8, 0, 4, 16, *ok_tail) == mpq.ERR_SHAPE
    assert f(FAKE, FAKE, 4, 4, 4, 15, *ok_tail) == mpq.ERR_SHAPE       # odd K with packed int4
    assert f(FAKE, FAKE, 8, 4, 4, 133144, *ok_tail) == mpq.ERR_SHAPE   # int32 could overflow
    assert f(FAKE, FAKE, 8, 4, 4, 16, FAKE, FAKE, 2, FAKE, None, None, 0, None) == mpq.ERR_GRAN
    assert f(FAKE, FAKE, 8, 4, 4, 16, FAKE, FAKE, 0, C.c_void_p(0x1002), None, None, 0, None) == mpq.ERR_ALIGN


@needs_no_gpu
def test_sse_pair_validation():
    L = mpq.lib()
    f = L.mpq_sse_pair
    need = L.mpq_sse_pair_workspace_bytes(1 << 20)
    assert need > 0 and L.mpq_sse_pair_workspace_bytes(0) == 0
    assert f(None, FAKE, 16, FAKE, FAKE16, need, None) == mpq.ERR_NULL
    assert f(FAKE, FAKE, 0, FAKE, FAKE16, need, None) == mpq.ERR_SHAPE
    assert f(FAKE16, FAKE16, 1 << 20, FAKE, None, 0, None) == mpq.ERR_WORKSPACE
    assert f(FAKE16, FAKE16, 1 << 20, FAKE, FAKE16, need - 8, None) == mpq.ERR_WORKSPACE


@needs_no_gpu
def test_qgemm_score_validation():
    L = mpq.lib()
    f = L.mpq_qgemm_score
    need = L.mpq_qgemm_score_workspace_bytes(256, 256, 64, 8)
    assert need == 16 * 8 and L.mpq_qgemm_score_workspace_bytes(0, 4, 4, 8) == 0
    head = (FAKE16, FAKE16, 8, 256, 256, 64, FAKE, FAKE, 0)
    assert f(*head, None, FAKE16, None, FAKE16, need, None) == mpq.ERR_NULL          # no y_ref
    assert f(*head, FAKE16, None, None, FAKE16, need, None) == mpq.ERR_NULL          # no sse_out
    assert f(*head, FAKE16, C.c_void_p(0x10004), None, FAKE16, need, None) == mpq.ERR_ALIGN
    assert f(*head, FAKE16, FAKE16, None, None, 0, None) == mpq.ERR_WORKSPACE
    assert f(*head, FAKE16, FAKE16, None, FAKE16, need - 8, None) == mpq.ERR_WORKSPACE
    assert f(FAKE16, FAKE16, 6, 256, 256, 64, FAKE, FAKE, 0, FAKE16, FAKE16, None, FAKE16, need, None) == mpq.ERR_BITS
    assert f(FAKE16, FAKE16, 8, 256, 256, 64, None, FAKE, 0, FAKE16, FAKE16, None, FAKE16, need, None) == mpq.ERR_NULL


@needs_no_gpu
def test_qgemm_act_and_act_codes_validation():
    L = mpq.lib()
    f = L.mpq_qgemm_act
    head = (FAKE16, FAKE16, 8, 256, 256, 64, FAKE, FAKE, 0)
    assert f(*head, 1, None, None, 0, None) == mpq.ERR_NULL                       # neither output
    assert f(*head, 3, FAKE16, None, 0, None) == mpq.ERR_SHAPE                    # unknown activation
    assert f(*head, 1, FAKE16, C.c_void_p(0x10002), 0, None) == mpq.ERR_ALIGN
    assert f(None, FAKE16, 8, 256, 256, 64, FAKE, FAKE, 0, 1, None, FAKE16, 0, None) == mpq.ERR_NULL
    assert f(FAKE16, FAKE16, 6, 256, 256, 64, FAKE, FAKE, 0, 1, None, FAKE16, 0, None) == mpq.ERR_BITS
    g = L.mpq_qgemm_act_codes
    assert g(*head, 1, None, 8, FAKE16, None) == mpq.ERR_NULL                     # no absmax
    assert g(*head, 1, FAKE16, 8, None, None) == mpq.ERR_NULL                     # no codes_out
    assert g(*head, 1, FAKE16, 9, FAKE16, None) == mpq.ERR_BITS
    assert g(*head, 1, FAKE16, 1, FAKE16, None) == mpq.ERR_BITS
    assert g(*head, 5, FAKE16, 8, FAKE16, None) == mpq.ERR_SHAPE
    assert g(*head, 1, C.c_void_p(0x10002), 8, FAKE16, None) == mpq.ERR_ALIGN
    assert g(FAKE16, FAKE16, 8, 256, 0, 64, FAKE, FAKE, 0, 1, FAKE16, 8, FAKE16, None) == mpq.ERR_SHAPE
    assert g(FAKE16, FAKE16, 8, 256, 256, 64, None, FAKE, 0, 1, FAKE16, 8, FAKE16, None) == mpq.ERR_NULL
    assert g(FAKE16, FAKE16, 4, 256, 256, 63, FAKE, FAKE, 0, 1, FAKE16, 8, FAKE16, None) == mpq.ERR_SHAPE


@needs_no_gpu
def test_hutchinson_validation_and_workspace_query():
    L = mpq.lib()
    r = L.mpq_rademacher
    assert r(1, 2, 4, 4, None, None) == mpq.ERR_NULL
    assert r(1, 2, 0, 4, FAKE16, None) == mpq.ERR_SHAPE
    assert r(1, 2, 1 << 20, 1 << 19, FAKE16, None) == mpq.ERR_SHAPE          # more than 2^38 elements
    f = L.mpq_hutchinson_quad
    need = L.mpq_hutchinson_quad_workspace_bytes(16384, 1024, 32)
    assert need >= 512 * 32 * 4 and L.mpq_hutchinson_quad_workspace_bytes(0, 4, 4) == 0
    assert L.mpq_hutchinson_quad_workspace_bytes(16384, 1024, 300) >= 512 * 64 * 4
    assert f(None, 64, 64, FAKE16, 32, FAKE16, FAKE16, need, None) == mpq.ERR_NULL
    assert f(FAKE16, 64, 64, None, 32, FAKE16, FAKE16, need, None) == mpq.ERR_NULL
    assert f(FAKE16, 64, 64, FAKE16, 32, None, FAKE16, need, None) == mpq.ERR_NULL
    assert f(FAKE16, 0, 64, FAKE16, 32, FAKE16, FAKE16, need, None) == mpq.ERR_SHAPE
    assert f(FAKE16, 64, 64, FAKE16, 0, FAKE16, FAKE16, need, None) == mpq.ERR_SHAPE
    assert f(FAKE16, 64, 64, FAKE16, (1 << 20) + 1, FAKE16, FAKE16, need, None) == mpq.ERR_SHAPE
    assert f(C.c_void_p(0x10002), 64, 64, FAKE16, 32, FAKE16, FAKE16, need, None) == mpq.ERR_ALIGN
    assert f(FAKE16, 64, 64, FAKE16, 32, C.c_void_p(0x10004), FAKE16, need, None) == mpq.ERR_ALIGN
    assert f(FAKE16, 16384, 1024, FAKE16, 32, FAKE16, None, 0, None) == mpq.ERR_WORKSPACE
    assert f(FAKE16, 16384, 1024, FAKE16, 32, FAKE16, FAKE16, need - 4, None) == mpq.ERR_WORKSPACE
    g = L.mpq_hutchinson_quad_signs
    assert g(None, 64, 64, 1, 2, 32, FAKE16, FAKE16, need, None) == mpq.ERR_NULL
    assert g(FAKE16, 64, 72, 1, 2, 32, FAKE16, FAKE16, need, None) == mpq.ERR_SHAPE       # K not a multiple of 16
    assert g(C.c_void_p(0x10004), 64, 64, 1, 2, 32, FAKE16, FAKE16, need, None) == mpq.ERR_SHAPE   # x not 16-byte aligned
    assert g(FAKE16, 16384, 1024, 1, 2, 32, FAKE16, FAKE16, need - 4, None) == mpq.ERR_WORKSPACE


@needs_no_gpu
def test_stack_evaluate_validation():
    L = mpq.lib()
    f = L.mpq_stack_evaluate
    nw = 2
    wq = (C.c_void_p * nw)(0x10000, 0x20000)
    wsc = (C.c_void_p * nw)(0x30000, 0x40000)
    st = (C.c_int * nw)(8, 4)

    def layer(N, K, h, store=st):
        return mpq.StackLayer(N, K, nw, C.cast(wq, C.POINTER(C.c_void_p)), C.cast(wsc, C.POINTER(C.c_void_p)),
                              C.cast(store, C.POINTER(C.c_int)), 0x50000, h)

    arr = (mpq.StackLayer * 2)(layer(64, 32, 0x60000), layer(16, 64, None))
    idx = (C.c_int * 2)(0, 1)
    need = L.mpq_stack_evaluate_workspace_bytes(arr, 2, 128)
    assert need == L.mpq_qgemm_score_workspace_bytes(128, 16, 64, 8) > 0
    tail = (FAKE16, FAKE16, FAKE16, FAKE16, FAKE16, need, None)
    assert f(None, 2, 128, idx, 8, 1, 0, *tail) == mpq.ERR_NULL
    assert f(arr, 2, 128, None, 8, 1, 0, *tail) == mpq.ERR_NULL
    assert f(arr, 0, 128, idx, 8, 1, 0, *tail) == mpq.ERR_SHAPE
    assert f(arr, 2, 128, idx, 9, 1, 0, *tail) == mpq.ERR_BITS
    assert f(arr, 2, 128, idx, 8, 7, 0, *tail) == mpq.ERR_SHAPE
    assert f(arr, 2, 128, (C.c_int * 2)(0, 2), 8, 1, 0, *tail) == mpq.ERR_SHAPE          # no such candidate width
    assert f(arr, 2, 128, idx, 8, 1, 0, FAKE16, FAKE16, FAKE16, FAKE16, FAKE16, need - 8, None) == mpq.ERR_WORKSPACE
    assert f(arr, 2, 128, idx, 8, 1, 0, FAKE16, FAKE16, None, FAKE16, FAKE16, need, None) == mpq.ERR_NULL
    broken = (mpq.StackLayer * 2)(layer(64, 32, 0x60000), layer(16, 48, None))            # 48 != 64: does not chain
    assert f(broken, 2, 128, idx, 8, 1, 0, *tail) == mpq.ERR_SHAPE
    no_h = (mpq.StackLayer * 2)(layer(64, 32, None), layer(16, 64, None))
    assert f(no_h, 2, 128, idx, 8, 1, 0, *tail) == mpq.ERR_NULL
    odd = (mpq.StackLayer * 1)(layer(16, 33, None))
    assert f(odd, 1, 128, (C.c_int * 1)(1), 8, 1, 0, *tail) == mpq.ERR_SHAPE               # packed nibbles need even K
    bad_store = (C.c_int * nw)(8, 6)
    assert f((mpq.StackLayer * 1)(layer(16, 32, None, bad_store)), 1, 128, (C.c_int * 1)(1), 8, 1, 0, *tail) == mpq.ERR_BITS


@needs_no_gpu
def test_scale_adjust_validation():
    L = mpq.lib()
    assert L.mpq_scale_grad_workspace_bytes(64, 64, 0) > 0
    assert L.mpq_scale_grad_workspace_bytes(64, 64, 1) == 0      # per row: results are written directly
    fq, sg, st = L.mpq_fake_quant_scales, L.mpq_scale_grad, L.mpq_scale_sgd_step
    assert fq(FAKE, 4, 4, 0, FAKE, FAKE, 4, None, None, None) == mpq.ERR_NULL
    assert fq(FAKE, 4, 4, 2, FAKE, FAKE, 4, FAKE, None, None) == mpq.ERR_GRAN   # per column is not offered
    assert fq(FAKE, 4, 4, 0, FAKE, FAKE, 9, FAKE, None, None) == mpq.ERR_BITS
    need = L.mpq_scale_grad_workspace_bytes(64, 64, 0)
    assert sg(FAKE16, 64, 64, 0, FAKE, FAKE, 4, None, None, FAKE16, None, FAKE16, need, None) == mpq.ERR_NULL
    assert sg(FAKE16, 64, 64, 0, FAKE, FAKE, 4, None, FAKE16, FAKE16, None, None, 0, None) == mpq.ERR_WORKSPACE
    assert sg(FAKE16, 64, 64, 0, FAKE, FAKE, 4, None, C.c_void_p(0x10004), FAKE16, None, FAKE16, need, None) == mpq.ERR_ALIGN
    assert sg(FAKE16, 0, 64, 0, FAKE, FAKE, 4, None, FAKE16, FAKE16, None, FAKE16, need, None) == mpq.ERR_SHAPE
    assert st(None, FAKE, FAKE, FAKE, 4, 1e-5, None) == mpq.ERR_NULL
    assert st(FAKE, FAKE, FAKE, FAKE, 0, 1e-5, None) == mpq.ERR_SHAPE


def test_python_errors_carry_the_message():
    with pytest.raises(mpq.MpqError) as e:
        mpq._check(mpq.ERR_BITS, "mpq_fake_quant")
    assert "bit-width" in str(e.value) and e.value.status == mpq.ERR_BITS


def _sweep_desc(x=0x10000, rows=8, cols=64, am_r=0x20000, am_t=0x30000, st=0x40000, sr=0x50000):
    return mpq.SweepTensor(x, rows, cols, am_r, am_t, st, sr)


def test_sweep_plan_build_validation_and_layout():
    """Pure host code: runs with or without a GPU (the pointers are never dereferenced)."""
    L = mpq.lib()
    arr = (mpq.SweepTensor * 2)(_sweep_desc(), _sweep_desc(rows=100, cols=4096))
    n = L.mpq_sweep_plan_bytes(arr, 2)
    assert n > 0 and L.mpq_sweep_plan_bytes(arr, 0) == 0 and L.mpq_sweep_plan_bytes(None, 2) == 0
    buf = (C.c_uint64 * ((n + 7) // 8))()
    assert L.mpq_sweep_plan_build(arr, 2, buf, n) == mpq.OK
    assert L.mpq_sweep_plan_build(arr, 2, buf, n - 1) == mpq.ERR_WORKSPACE
    assert L.mpq_sweep_plan_build(None, 2, buf, n) == mpq.ERR_NULL
    assert L.mpq_sweep_plan_build(arr, 2, None, n) == mpq.ERR_NULL
    assert L.mpq_sweep_plan_build(arr, 0, buf, n) == mpq.ERR_SHAPE
    # per-tensor workspace: one partial per 64 K-element chunk and bit-width (1 + 7 chunks here)
    assert L.mpq_quant_error_batch_workspace_bytes(buf, mpq.PER_TENSOR, 2, 8) == (1 + 7) * 7 * 8
    assert L.mpq_quant_error_batch_workspace_bytes(buf, mpq.PER_ROW, 2, 8) == 0
    assert L.mpq_quant_error_batch_workspace_bytes(buf, mpq.SWEEP_TENSOR_AND_ROW, 2, 8) > 0
    assert L.mpq_quant_error_batch_workspace_bytes(buf, mpq.PER_TENSOR, 1, 8) == 0
    for bad, want in ((_sweep_desc(x=0), mpq.ERR_NULL), (_sweep_desc(x=0x10004), mpq.ERR_ALIGN),
                      (_sweep_desc(cols=66), mpq.ERR_SHAPE), (_sweep_desc(rows=0), mpq.ERR_SHAPE),
                      (_sweep_desc(cols=16388), mpq.ERR_SHAPE), (_sweep_desc(am_r=0), mpq.ERR_NULL),
                      (_sweep_desc(am_t=0), mpq.ERR_NULL), (_sweep_desc(st=0x40004), mpq.ERR_ALIGN)):
        one = (mpq.SweepTensor * 1)(bad)
        assert L.mpq_sweep_plan_build(one, 1, buf, n) == want


@needs_no_gpu
def test_sweep_batch_call_validation():
    L = mpq.lib()
    arr = (mpq.SweepTensor * 1)(_sweep_desc())
    n = L.mpq_sweep_plan_bytes(arr, 1)
    buf = (C.c_uint64 * ((n + 7) // 8))()
    assert L.mpq_sweep_plan_build(arr, 1, buf, n) == mpq.OK
    junk = (C.c_uint64 * 8)()
    assert L.mpq_calibrate_absmax_batch(junk, FAKE16, None) == mpq.ERR_SHAPE      # not a plan
    assert L.mpq_calibrate_absmax_batch(buf, None, None) == mpq.ERR_NULL
    assert L.mpq_calibrate_absmax_batch(buf, C.c_void_p(0x10004), None) == mpq.ERR_ALIGN
    f = L.mpq_quant_error_batch
    assert f(buf, FAKE16, mpq.PER_COL, 2, 8, FAKE16, 1 << 20, None) == mpq.ERR_GRAN
    assert f(buf, FAKE16, mpq.PER_TENSOR, 2, 9, FAKE16, 1 << 20, None) == mpq.ERR_BITS
    assert f(buf, FAKE16, mpq.PER_TENSOR, 2, 8, None, 0, None) == mpq.ERR_WORKSPACE
    assert f(buf, FAKE16, mpq.PER_TENSOR, 2, 8, FAKE16, 8, None) == mpq.ERR_WORKSPACE
    nost = (mpq.SweepTensor * 1)(_sweep_desc(st=0))
    assert L.mpq_sweep_plan_build(nost, 1, buf, n) == mpq.OK
    assert f(buf, FAKE16, mpq.PER_TENSOR, 2, 8, FAKE16, 1 << 20, None) == mpq.ERR_NULL
    # the one-read form of calibration + per-row sums
    g = L.mpq_calibrate_quant_error_rows_batch
    assert g(junk, FAKE16, 2, 8, None) == mpq.ERR_SHAPE
    assert g(buf, None, 2, 8, None) == mpq.ERR_NULL
    assert g(buf, C.c_void_p(0x10004), 2, 8, None) == mpq.ERR_ALIGN
    assert g(buf, FAKE16, 1, 8, None) == mpq.ERR_BITS
    assert g(buf, FAKE16, 5, 4, None) == mpq.ERR_BITS
    nosr = (mpq.SweepTensor * 1)(_sweep_desc(sr=0))
    assert L.mpq_sweep_plan_build(nosr, 1, buf, n) == mpq.OK
    assert g(buf, FAKE16, 2, 8, None) == mpq.ERR_NULL


@needs_no_gpu
def test_quantized_layer_calls_check_everything_before_their_first_launch():
    """mpq_qgemm_act clears the running maximum with a small kernel before the product: every argument
    error -- also the ones the shared dispatcher used to find only afterwards -- has to be reported
    before that kernel could be enqueued.  (Without a GPU any launch attempt would surface as
    MPQ_ERR_HIP instead of the argument error expected here.)"""
    L = mpq.lib()
    f = L.mpq_qgemm_act
    ok = dict(a=FAKE16, w=FAKE16, bits=8, M=64, N=64, K=64, sa=FAKE16, sw=FAKE16, gran=mpq.PER_TENSOR, act=1,
              y=FAKE16, am=FAKE16, acc=0)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["a"], a["w"], a["bits"], a["M"], a["N"], a["K"], a["sa"], a["sw"], a["gran"], a["act"], a["y"], a["am"],
                 a["acc"], None)

    assert call(y=C.c_void_p(0x10002)) == mpq.ERR_ALIGN            # 4-byte alignment of the output
    assert call(am=C.c_void_p(0x10002)) == mpq.ERR_ALIGN
    assert call(M=1 << 40, N=1 << 40) == mpq.ERR_SHAPE              # M * N overflows the element limit
    assert call(M=70000 * 128 + 1, N=64) == mpq.ERR_SHAPE           # more row tiles than a grid holds
    assert call(K=133144) == mpq.ERR_SHAPE
    assert call(bits=4, K=63) == mpq.ERR_SHAPE
    assert call(gran=mpq.PER_COL) == mpq.ERR_GRAN
    assert call(act=7) == mpq.ERR_SHAPE
    assert call(sa=None) == mpq.ERR_NULL
    assert call(y=None, am=None) == mpq.ERR_NULL
    # the stack evaluator applies the same per-layer checks to ALL layers before its clearing kernel
    wq = (C.c_void_p * 1)(0x10000)
    wsc = (C.c_void_p * 1)(0x20000)
    st = (C.c_int * 1)(8)
    good = mpq.StackLayer(64, 64, 1, C.cast(wq, C.POINTER(C.c_void_p)), C.cast(wsc, C.POINTER(C.c_void_p)),
                          C.cast(st, C.POINTER(C.c_int)), 0x30000, 0x40000)
    bad_k = mpq.StackLayer(64, 133144, 1, C.cast(wq, C.POINTER(C.c_void_p)), C.cast(wsc, C.POINTER(C.c_void_p)),
                           C.cast(st, C.POINTER(C.c_int)), 0x30000, None)
    misaligned_h = mpq.StackLayer(64, 64, 1, C.cast(wq, C.POINTER(C.c_void_p)), C.cast(wsc, C.POINTER(C.c_void_p)),
                                  C.cast(st, C.POINTER(C.c_int)), 0x30000, 0x40002)
    last = mpq.StackLayer(64, 64, 1, C.cast(wq, C.POINTER(C.c_void_p)), C.cast(wsc, C.POINTER(C.c_void_p)),
                          C.cast(st, C.POINTER(C.c_int)), 0x30000, None)
    idx = (C.c_int * 3)(0, 0, 0)
    g = L.mpq_stack_evaluate
    for layers, want in (((good, misaligned_h, last), mpq.ERR_ALIGN), ((good, good, bad_k), mpq.ERR_SHAPE)):
        arr = (mpq.StackLayer * 3)(*layers)
        assert g(arr, 3, 64, idx, 8, 1, mpq.PER_TENSOR, FAKE16, FAKE16, FAKE16, FAKE16, FAKE16, 1 << 20, None) == want
