"""Parity of the HIP library with the CPU oracle, element by element, on identical seeded inputs.
Bit-exact: absmax, codes, packed nibbles, int32 accumulators, noise.  Tolerances: dequantized
values 1e-5 relative, error sums 1e-4 relative."""
import numpy as np
import pytest

import oracle
from paper_2302_01382_amd import mpq, workloads

pytestmark = pytest.mark.gpu

GRANS = [mpq.PER_TENSOR, mpq.PER_ROW, mpq.PER_COL]
# several tiles + ragged tails; odd sizes force the scalar / generic paths
SHAPES = [(64, 256), (37, 53), (1, 1), (3, 7), (257, 1028), (5, 70004), (1031, 12), (2, 40000)]
RTOL_Y, RTOL_SSE = 1e-5, 1e-4


def torch():
    import torch as t
    return t


def dev(a):
    return torch().from_numpy(np.ascontiguousarray(a)).cuda()


def dev_misaligned(a):
    """Same values at a device address that is 4 bytes past a 16-byte boundary."""
    t = torch()
    flat = t.empty(a.size + 1, dtype=t.from_numpy(a).dtype, device="cuda")
    view = flat[1:].view(a.shape)
    view.copy_(t.from_numpy(np.ascontiguousarray(a)))
    return view


def host(t):
    torch().cuda.synchronize()
    return t.cpu().numpy()


def data(shape, seed, sigma=1.0):
    r = np.random.Generator(np.random.PCG64(seed))
    x = (sigma * r.standard_normal(shape)).astype(np.float32)
    if x.size > 8:
        x.ravel()[r.integers(0, x.size, 3)] *= np.float32(6.0)  # a few outliers
    return x


# ----------------------------------------------------------------------------------- absmax
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("gran", GRANS)
def test_absmax_bit_exact(shape, gran):
    x = data(shape, 1)
    want = oracle.absmax(x, gran)
    for mk in (dev, dev_misaligned):
        got = host(mpq.calibrate_absmax(mk(x), gran))
        np.testing.assert_array_equal(got, want)


def test_absmax_running_max_and_zero_tensor():
    x1, x2 = data((129, 260), 2), data((129, 260), 3, 2.0)
    for gran in GRANS:
        out = mpq.calibrate_absmax(dev(x1), gran)
        mpq.calibrate_absmax(dev(x2), gran, out=out, accumulate=True)
        want = oracle.absmax(x2, gran, running=oracle.absmax(x1, gran))
        np.testing.assert_array_equal(host(out), want)
    z = np.zeros((16, 16), np.float32)
    assert host(mpq.calibrate_absmax(dev(z)))[0] == 0.0
    # overwrite mode really overwrites a stale, larger value
    out = dev(np.array([1e30], np.float32))
    mpq.calibrate_absmax(dev(x1), mpq.PER_TENSOR, out=out)
    assert host(out)[0] == oracle.absmax(x1)[0]


def test_scale_from_absmax_bit_exact():
    am = np.array([0.0, 1.0, 0.2, 3.75, 1e-3, 117.25, 7.0], np.float32)
    for b in range(2, 9):
        np.testing.assert_array_equal(host(mpq.scale_from_absmax(dev(am), b)), oracle.scale_from_absmax(am, b))


# -------------------------------------------------------------------------------- fake quant
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("gran", GRANS)
def test_fake_quant_codes_bit_exact_all_bits(shape, gran):
    x = data(shape, 4)
    am = oracle.absmax(x, gran)
    for bits in range(2, 9):
        packed_ok = bits <= 4 and shape[1] % 2 == 0
        y_o, c_o, p_o = oracle.fake_quant(x, am, bits, gran, want_packed4=packed_ok)
        for mk in (dev, dev_misaligned):
            y, c, p = mpq.fake_quant(mk(x), dev(am), bits, gran, want_y=True, want_codes=True,
                                     want_packed4=packed_ok)
            np.testing.assert_array_equal(host(c), c_o)
            np.testing.assert_allclose(host(y), y_o, rtol=RTOL_Y, atol=0)
            if packed_ok:
                np.testing.assert_array_equal(host(p), p_o)


@pytest.mark.parametrize("shape", [(1, 1), (7, 13), (64, 256), (300, 1030)])
def test_fake_quant_step_is_fake_quant_plus_the_step_size(shape):
    x = data(shape, 33)
    am_o = oracle.absmax(x)
    for mk in (dev, dev_misaligned):
        dx = mk(x)
        am = mpq.calibrate_absmax(dx)
        for bits in (2, 4, 8):
            y, codes, _, step = mpq.fake_quant_step(dx, am, bits, want_codes=True)
            y_o, c_o, _ = oracle.fake_quant(x, am_o, bits)
            np.testing.assert_array_equal(host(codes), c_o)
            np.testing.assert_allclose(host(y), y_o, rtol=RTOL_Y, atol=0)
            np.testing.assert_array_equal(host(step), oracle.scale_from_absmax(am_o, bits))
            np.testing.assert_array_equal(host(step), host(mpq.scale_from_absmax(am, bits)))
    if shape[1] % 2 == 0:
        _, _, packed, step = mpq.fake_quant_step(dev(x), dev(am_o), 4, want_y=False, want_packed4=True)
        _, _, p_o = oracle.fake_quant(x, am_o, 4, want_packed4=True)
        np.testing.assert_array_equal(host(packed), p_o)
        np.testing.assert_array_equal(host(step), oracle.scale_from_absmax(am_o, 4))


def test_fake_quant_saturation_zero_channels_and_single_outputs():
    x = data((130, 516), 5)
    for gran in GRANS:
        am = oracle.absmax(x, gran) * np.float32(0.3)   # most values beyond the range
        if am.size > 2:
            am[1] = 0.0                                  # an all-zero-scale channel
        for bits in (2, 4, 8):
            y_o, c_o, p_o = oracle.fake_quant(x, am, bits, gran, want_packed4=bits <= 4)
            y, _, _ = mpq.fake_quant(dev(x), dev(am), bits, gran, want_y=True)
            np.testing.assert_allclose(host(y), y_o, rtol=RTOL_Y, atol=0)
            _, c, _ = mpq.fake_quant(dev(x), dev(am), bits, gran, want_y=False, want_codes=True)
            np.testing.assert_array_equal(host(c), c_o)
            assert np.abs(host(c)).max() == oracle.qmax(bits)
            if bits <= 4:
                _, _, p = mpq.fake_quant(dev(x), dev(am), bits, gran, want_y=False, want_packed4=True)
                np.testing.assert_array_equal(host(p), p_o)


def test_fake_quant_ties_follow_round_half_even():
    for bits in range(2, 9):
        q = oracle.qmax(bits)
        x = (np.arange(-2 * q - 1, 2 * q + 2, dtype=np.float32) * np.float32(0.5)).reshape(1, -1)
        x = np.concatenate([x, x], 1)[:, : (x.shape[1] * 2) // 4 * 4]
        am = np.array([q], np.float32)  # inv = scale = 1: every half-integer is an exact tie
        _, c_o, _ = oracle.fake_quant(x, am, bits)
        _, c, _ = mpq.fake_quant(dev(x), dev(am), bits, want_y=False, want_codes=True)
        np.testing.assert_array_equal(host(c), c_o)


# ------------------------------------------------------------------------------- quant error
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("gran", GRANS)
def test_quant_error_sweep(shape, gran):
    x = data(shape, 6)
    am = oracle.absmax(x, gran)
    want = oracle.quant_error(x, am, 2, 8, gran)
    for mk in (dev, dev_misaligned):
        got = host(mpq.quant_error(mk(x), dev(am), 2, 8, gran))
        assert got.shape == want.shape
        np.testing.assert_allclose(got, want, rtol=RTOL_SSE, atol=1e-30)


def test_quant_error_sub_ranges_foreign_absmax_and_reproducibility():
    x = data((300, 1028), 7)
    for gran in GRANS:
        am = oracle.absmax(x, gran) * np.float32(0.5)  # clipping contributes to the error
        if am.size > 3:
            am[2] = 0.0
        for lo, hi in ((2, 8), (3, 5), (8, 8), (2, 2), (4, 8)):
            want = oracle.quant_error(x, am, lo, hi, gran)
            got = host(mpq.quant_error(dev(x), dev(am), lo, hi, gran))
            np.testing.assert_allclose(got, want, rtol=RTOL_SSE, atol=1e-30)
        a = host(mpq.quant_error(dev(x), dev(am), 2, 8, gran))
        b = host(mpq.quant_error(dev(x), dev(am), 2, 8, gran))
        np.testing.assert_array_equal(a, b)  # fixed combination order: same bits every run



def test_quant_error_of_a_tensor_on_the_grid_is_exactly_zero():
    """Eq. 2 over the reals: a tensor made of grid points code * scale_b has SSE_b == 0.  With a
    power-of-two step the tensor is exact in fp32 and both sides must return 0.0, not 1e-15."""
    r = np.random.Generator(np.random.PCG64(31))
    for b in range(2, 9):
        q = (1 << (b - 1)) - 1
        codes = r.integers(-q, q + 1, size=(301, 1028))
        codes[0, 0] = q
        x = (codes * np.float32(2.0 ** -5)).astype(np.float32)
        for gran in GRANS:
            am = oracle.absmax(x, gran)
            keep = am == np.float32(q * 2.0 ** -5)              # channels whose maximum code is qmax
            want = oracle.quant_error(x, am, 2, 8, gran)
            got = host(mpq.quant_error(dev(x), dev(am), 2, 8, gran))
            assert np.all(want[keep, b - 2] == 0.0) and np.all(got[keep, b - 2] == 0.0)
            np.testing.assert_allclose(got, want, rtol=RTOL_SSE, atol=1e-30)
    # full-mantissa step: the sum of squared product roundings, tiny but not zero, on both sides
    am = np.array([0.7321], np.float32)
    s8 = oracle.scale_from_absmax(am, 8)[0]
    x = (r.integers(-127, 128, size=(300, 1028)).astype(np.float32) * s8).astype(np.float32)
    want = oracle.quant_error(x, am, 8, 8)
    assert 0.0 < want[0, 0] < 1e-9
    np.testing.assert_allclose(host(mpq.quant_error(dev(x), dev(am), 8, 8)), want, rtol=RTOL_SSE, atol=0)


def test_quant_error_argmin_bit_selection_matches_oracle():
    """Smallest b whose E_QE (Eq. 2) is below a threshold, and the ordering of tensors by E_QE."""
    tensors = [data((64, 256), 20 + i, s) for i, s in enumerate((1.0, 0.05, 3.0, 0.5))]
    tensors[2].ravel()[5] = 200.0  # one tensor dominated by an outlier
    e_or, e_gpu = [], []
    for x in tensors:
        am = oracle.absmax(x)
        so = oracle.quant_error(x, am)[0]
        sg = host(mpq.quant_error(dev(x), mpq.calibrate_absmax(dev(x))))[0]
        e_or.append([oracle.eqe(s, x.size, float(am[0])) for s in so])
        e_gpu.append([oracle.eqe(s, x.size, float(am[0])) for s in sg])
    e_or, e_gpu = np.array(e_or), np.array(e_gpu)
    for tau in (0.3, 0.1, 0.03, 0.01, 0.003):
        margin = np.abs(e_or - tau) / tau
        pick = lambda e: [next((b for b in range(7) if row[b] <= tau), 6) + 2 for row in e]
        if margin.min() > 2e-4:  # decision not within the error-sum tolerance of the threshold
            assert pick(e_gpu) == pick(e_or)
    for b in range(7):
        col = np.sort(e_or[:, b])
        if np.min(np.diff(col) / col[:-1]) > 2e-4:
            assert np.argsort(e_gpu[:, b], kind="stable").tolist() == np.argsort(e_or[:, b], kind="stable").tolist()


# ------------------------------------------------------------------------------------- noise
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("gran", GRANS)
def test_noise_bit_exact(shape, gran):
    x = data(shape, 8)
    am = oracle.absmax(x, gran)
    for bits, lam, seed, sid in ((4, 0.28867513, 0, 0), (8, 1.0, 0xDEADBEEFCAFEF00D, 2 ** 40 + 3)):
        want = oracle.noise_inject(x, am, bits, lam, seed, sid, gran)
        for mk in (dev, dev_misaligned):
            got = host(mpq.noise_inject(mk(x), dev(am), bits, lam, seed, sid, gran))
            np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("gran", GRANS)
def test_noise_sweep_planes_equal_single_calls_bit_exact(shape, gran):
    x = data(shape, 8)
    am = oracle.absmax(x, gran)
    t = torch()
    for (b_lo, b_hi), lam, seed, sid in (((2, 8), 0.28867513, 7, 1), ((4, 5), 1.0, 0xDEADBEEFCAFEF00D, 2 ** 40 + 3)):
        want = oracle.noise_inject_sweep(x, am, b_lo, b_hi, lam, seed, sid, gran)
        nb = b_hi - b_lo + 1
        for mk in (dev, dev_misaligned):
            got = host(mpq.noise_inject_sweep(mk(x), dev(am), b_lo, b_hi, lam, seed, sid, gran))
            np.testing.assert_array_equal(got, want)
        # planes further apart than one tensor (and not a multiple of 4 elements apart)
        buf = t.full((nb, x.size + 3), -1.0, dtype=t.float32, device="cuda")
        out = buf.as_strided((nb,) + x.shape, (x.size + 3, x.shape[1], 1))
        mpq.noise_inject_sweep(dev(x), dev(am), b_lo, b_hi, lam, seed, sid, gran, out=out)
        np.testing.assert_array_equal(host(out), want)
        assert (host(buf)[:, x.size:] == -1.0).all()   # the gaps between planes are left alone


def test_noise_standard_normals_bit_exact_on_a_large_sample():
    n = 1 << 21
    zero = np.zeros((512, n // 512), np.float32)
    am = np.array([7.0], np.float32)   # b = 4 -> scale 1, lambda 1: output is z itself
    want = oracle.noise_inject(zero, am, 4, 1.0, 123, 9)
    got = host(mpq.noise_inject(dev(zero), dev(am), 4, 1.0, 123, 9))
    np.testing.assert_array_equal(got, want)
    # in place is allowed
    t = dev(zero)
    mpq.noise_inject(t, dev(am), 4, 1.0, 123, 9, out=t)
    np.testing.assert_array_equal(host(t), want)


# ------------------------------------------------------------------------------------- qgemm
GEMM_SHAPES = [(64, 256, 256), (1, 1, 2), (33, 31, 130), (129, 257, 64), (128, 128, 4608),
               (300, 70, 48), (257, 129, 1000), (2, 3, 18)]


def rand_codes(shape, q, seed):
    r = np.random.Generator(np.random.PCG64(seed))
    return r.integers(-q, q + 1, shape).astype(np.int8)


@pytest.mark.parametrize("mnk", GEMM_SHAPES)
def test_qgemm_int8_accumulators_bit_exact(mnk):
    M, N, K = mnk
    a, w = rand_codes((M, K), 127, 9), rand_codes((N, K), 127, 10)
    sa = np.array([0.0123], np.float32)
    sw = (np.random.Generator(np.random.PCG64(11)).random(N).astype(np.float32) + 0.5) * np.float32(1e-3)
    for gran, s in ((mpq.PER_TENSOR, sw[:1]), (mpq.PER_ROW, sw)):
        y_o, acc_o = oracle.qgemm(a, w, sa, s, 8, gran)
        for mk in (dev, dev_misaligned):
            y, acc = mpq.qgemm(mk(a), mk(w), dev(sa), dev(s), 8, gran, want_y=True, want_acc=True)
            np.testing.assert_array_equal(host(acc), acc_o)
            np.testing.assert_allclose(host(y), y_o, rtol=RTOL_Y, atol=0)


@pytest.mark.parametrize("mnk", GEMM_SHAPES)
def test_qgemm_packed_int4_weights_bit_exact(mnk):
    M, N, K = mnk
    a, w = rand_codes((M, K), 127, 12), rand_codes((N, K), 7, 13)
    w[0, 0] = -7
    wp = oracle.pack4(w)
    sa, sw = np.array([0.5], np.float32), np.array([0.031], np.float32)
    y_o, acc_o = oracle.qgemm(a, wp, sa, sw, 4)
    for mk in (dev, dev_misaligned):
        y, acc = mpq.qgemm(mk(a), mk(wp), dev(sa), dev(sw), 4, want_y=True, want_acc=True)
        np.testing.assert_array_equal(host(acc), acc_o)
        np.testing.assert_allclose(host(y), y_o, rtol=RTOL_Y, atol=0)
    # the same codes stored as int8 give the same result
    _, acc8 = mpq.qgemm(dev(a), dev(w), dev(sa), dev(sw), 8, want_y=False, want_acc=True)
    np.testing.assert_array_equal(host(acc8), acc_o)


@pytest.mark.parametrize("mnk,wbits", [((4096, 4096, 256), 8), ((4100, 4092, 160), 4), ((2048, 2048, 384), 8),
                                        ((2085, 2047, 96), 4), ((2085, 2046, 112), 8), ((16384, 1024, 4096), 8),
                                        ((1568, 2048, 2048), 4), ((1568, 512, 4608), 8), ((300, 200, 1152), 4),
                                        ((12288, 768, 256), 8), ((12288, 768, 1152), 4), ((12280, 768, 160), 8)])
def test_qgemm_large_tiles_on_sampled_rows(mnk, wbits):
    """Shapes that select the 128 x 128, 192 x 192 and 256 x 256 tiles (ragged edges, N not a multiple of 4);
    rows of the product are independent, so the oracle checks a sample of rows exactly."""
    M, N, K = mnk
    q = 127 if wbits == 8 else 7
    a, w = rand_codes((M, K), 127, 30), rand_codes((N, K), q, 31)
    ws = w if wbits == 8 else oracle.pack4(w)
    sa = np.array([0.02], np.float32)
    sw = (np.random.Generator(np.random.PCG64(32)).random(N).astype(np.float32) + 0.5) * np.float32(1e-3)
    y, acc = mpq.qgemm(dev(a), dev(ws), dev(sa), dev(sw), wbits, mpq.PER_ROW, want_y=True, want_acc=True)
    r = np.random.Generator(np.random.PCG64(33))
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 63, 64, 127, 128, 255, 256, M - 257, M - 129, M - 2, M - 1],
                                     r.integers(0, M, 40)]))
    y_o, acc_o = oracle.qgemm(a[rows], ws, sa, sw, wbits, oracle.PER_ROW)
    np.testing.assert_array_equal(host(acc)[rows], acc_o)
    np.testing.assert_allclose(host(y)[rows], y_o, rtol=RTOL_Y, atol=0)
    # every row against a wide-integer matmul on the device side of torch would be plumbing; a
    # cheap global invariant instead: column sums of acc equal (sum of A rows) . W
    colsum = a.astype(np.int64).sum(0) @ w.astype(np.int64).T
    np.testing.assert_array_equal(host(acc).astype(np.int64).sum(0), colsum)
    # per-channel scales or an output that are only 4-byte aligned take the scalar epilogue: same bits
    y_s, _ = mpq.qgemm(dev(a), dev(ws), dev(sa), dev_misaligned(sw), wbits, mpq.PER_ROW)
    np.testing.assert_array_equal(host(y_s), host(y))
    y_buf = dev_misaligned(np.zeros((M, N), np.float32))
    mpq.qgemm(dev(a), dev(ws), dev(sa), dev(sw), wbits, mpq.PER_ROW, y=y_buf)
    np.testing.assert_array_equal(host(y_buf), host(y))
    # one scale for the whole weight tensor
    y_t, _ = mpq.qgemm(dev(a), dev(ws), dev(sa), dev(sw[:1].copy()), wbits, mpq.PER_TENSOR)
    y_to, _ = oracle.qgemm(a[rows], ws, sa, sw[:1], wbits, oracle.PER_TENSOR)
    np.testing.assert_allclose(host(y_t)[rows], y_to, rtol=RTOL_Y, atol=0)


@pytest.mark.parametrize("mnk,wbits", [((200, 130, 4608), 8), ((200, 132, 4608), 4), ((49, 512, 4608), 8),
                                        ((49, 512, 2048), 4), ((130, 70, 1040), 8), ((300, 200, 1056), 4),
                                        ((70, 131, 2048), 8), ((1, 64, 16384), 8), ((64, 1000, 1024), 4),
                                        ((500, 500, 1152), 8)])
def test_qgemm_split_along_k_is_bit_identical(mnk, wbits):
    """Few output tiles and a long K: with a workspace the library cuts K into ranges (ragged last
    range, K not a multiple of the k tile or of the range count, packed int4, N not a multiple of
    4) and adds the integer partial products.  Accumulators equal the oracle's bit for bit, Y to
    1e-5, and both equal the unsplit run of the same call."""
    M, N, K = mnk
    assert mpq.qgemm_workspace_bytes(M, N, K, wbits) >= 2 * 4 * M * N       # this shape is split
    q = 127 if wbits == 8 else 7
    a, w = rand_codes((M, K), 127, 60), rand_codes((N, K), q, 61)
    ws = w if wbits == 8 else oracle.pack4(w)
    sa = np.array([0.02], np.float32)
    sw = (np.random.Generator(np.random.PCG64(62)).random(N).astype(np.float32) + 0.5) * np.float32(1e-3)
    y_o, acc_o = oracle.qgemm(a, ws, sa, sw, wbits, oracle.PER_ROW)
    y, acc = mpq.qgemm(dev(a), dev(ws), dev(sa), dev(sw), wbits, mpq.PER_ROW, want_y=True, want_acc=True)
    np.testing.assert_array_equal(host(acc), acc_o)
    np.testing.assert_allclose(host(y), y_o, rtol=RTOL_Y, atol=0)
    y1, acc1 = mpq.qgemm(dev(a), dev(ws), dev(sa), dev(sw), wbits, mpq.PER_ROW, want_y=True, want_acc=True,
                         use_workspace=False)
    np.testing.assert_array_equal(host(acc1), host(acc))
    np.testing.assert_array_equal(host(y1), host(y))
    # outputs and scales that are only 4-byte aligned take the scalar combine: same bits
    y_buf = dev_misaligned(np.zeros((M, N), np.float32))
    acc_buf = dev_misaligned(np.zeros((M, N), np.int32))
    mpq.qgemm(dev(a), dev(ws), dev(sa), dev_misaligned(sw), wbits, mpq.PER_ROW, y=y_buf, acc=acc_buf)
    np.testing.assert_array_equal(host(y_buf), host(y))
    np.testing.assert_array_equal(host(acc_buf), acc_o)
    # a single output, one scale for the tensor
    y_t, none = mpq.qgemm(dev(a), dev(ws), dev(sa), dev(sw[:1].copy()), wbits, mpq.PER_TENSOR)
    assert none is None
    np.testing.assert_allclose(host(y_t), oracle.qgemm(a, ws, sa, sw[:1], wbits, oracle.PER_TENSOR)[0], rtol=RTOL_Y, atol=0)


def test_qgemm_extreme_operands_and_single_outputs():
    a = np.full((130, 4608), -127, np.int8)
    w = np.full((70, 4608), 127, np.int8)
    a[::2] = 127
    _, acc_o = oracle.qgemm(a, w, [1.0], [1.0])
    _, acc = mpq.qgemm(dev(a), dev(w), None, None, want_y=False, want_acc=True)
    np.testing.assert_array_equal(host(acc), acc_o)
    assert abs(int(host(acc)[0, 0])) == 4608 * 127 * 127
    s = dev(np.array([1.0], np.float32))
    y, none = mpq.qgemm(dev(a), dev(w), s, s, want_y=True, want_acc=False)
    assert none is None
    np.testing.assert_array_equal(host(y), acc_o.astype(np.float32))
    w4 = np.full((70, 4608), -8, np.int8)   # the nibble -8 is decodable even if never produced
    _, acc4o = oracle.qgemm(a, oracle.pack4(w4), [1.0], [1.0], 4)
    _, acc4 = mpq.qgemm(dev(a), dev(oracle.pack4(w4)), None, None, 4, want_y=False, want_acc=True)
    np.testing.assert_array_equal(host(acc4), acc4o)


# ------------------------------------------------------------------------------ qgemm + score
def score_case(M, N, K, wbits, gran, seed):
    q = 127 if wbits == 8 else 7
    a, w = rand_codes((M, K), 127, seed), rand_codes((N, K), q, seed + 1)
    ws = w if wbits == 8 else oracle.pack4(w)
    r = np.random.Generator(np.random.PCG64(seed + 2))
    sa = np.array([0.02], np.float32)
    sw = (r.random(N if gran == mpq.PER_ROW else 1).astype(np.float32) + 0.5) * np.float32(1e-3)
    y_o, _ = oracle.qgemm(a, ws, sa, sw, wbits, gran)
    # a reference output near the quantized one, as the fp32 layer output is in a search
    y_ref = (y_o + np.float32(0.05) * np.abs(y_o).mean() * r.standard_normal(y_o.shape)).astype(np.float32)
    return a, ws, sa, sw, y_o, y_ref, oracle.sse_pair(y_o, y_ref)


@pytest.mark.parametrize("mnk", GEMM_SHAPES)
@pytest.mark.parametrize("wbits", [8, 4])
def test_qgemm_score_small_shapes(mnk, wbits):
    M, N, K = mnk
    if wbits == 4 and K % 2:
        pytest.skip("packed int4 needs an even K")
    for gran in (mpq.PER_TENSOR, mpq.PER_ROW):
        a, ws, sa, sw, y_o, y_ref, want = score_case(M, N, K, wbits, gran, 40)
        for mk in (dev, dev_misaligned):   # the misaligned copies take the byte-wise kernel
            sse, y = mpq.qgemm_score(mk(a), mk(ws), dev(sa), dev(sw), mk(y_ref), wbits, gran, want_y=True)
            assert host(sse)[0] == pytest.approx(want, rel=RTOL_SSE)
            np.testing.assert_allclose(host(y), y_o, rtol=RTOL_Y, atol=0)
            sse2, none = mpq.qgemm_score(mk(a), mk(ws), dev(sa), dev(sw), mk(y_ref), wbits, gran)
            assert none is None
            assert host(sse2)[0] == host(sse)[0]   # same kernel, same order: reproducible


@pytest.mark.parametrize("mnk,wbits", [((2048, 2048, 384), 8), ((4100, 4092, 160), 4), ((2085, 2046, 112), 8),
                                        ((300, 200, 1152), 4), ((1568, 512, 1024), 8), ((6272, 256, 512), 4),
                                        ((12288, 768, 128), 8), ((130, 70, 1296), 8), ((100, 200, 2080), 4)])
def test_qgemm_score_every_tile_size(mnk, wbits):
    """Shapes that select the 64 (k tiles of 128 and of 256 bytes), 128 and 256 tiles, with ragged edges, N
    not a multiple of 4 and several tiles per workgroup; the whole product is small enough for the oracle."""
    M, N, K = mnk
    a, ws, sa, sw, y_o, y_ref, want = score_case(M, N, K, wbits, mpq.PER_ROW, 50)
    da, dw, dsa, dsw, dref = dev(a), dev(ws), dev(sa), dev(sw), dev(y_ref)
    sse, none = mpq.qgemm_score(da, dw, dsa, dsw, dref, wbits, mpq.PER_ROW)
    assert none is None
    assert host(sse)[0] == pytest.approx(want, rel=RTOL_SSE)
    sse_y, y = mpq.qgemm_score(da, dw, dsa, dsw, dref, wbits, mpq.PER_ROW, want_y=True)
    assert host(sse_y)[0] == pytest.approx(want, rel=RTOL_SSE)
    np.testing.assert_allclose(host(y), y_o, rtol=RTOL_Y, atol=0)
    # y_ref == the layer's own output: the score is exactly zero
    zero, _ = mpq.qgemm_score(da, dw, dsa, dsw, y, wbits, mpq.PER_ROW)
    assert host(zero)[0] == 0.0
    # a y_ref that is only 4-byte aligned takes the scalar epilogue
    sse_m, _ = mpq.qgemm_score(da, dw, dsa, dsw, dev_misaligned(y_ref), wbits, mpq.PER_ROW)
    assert host(sse_m)[0] == pytest.approx(want, rel=RTOL_SSE)


# ------------------------------------------------------------------- qgemm + activation + absmax
@pytest.mark.parametrize("mnk,wbits", [((64, 256, 256), 8), ((33, 31, 130), 8), ((300, 70, 48), 4), ((2048, 2048, 384), 8),
                                        ((4100, 4092, 160), 4), ((2085, 2046, 112), 8), ((6272, 256, 512), 4),
                                        ((12288, 768, 128), 4), ((130, 70, 1296), 8), ((100, 200, 2080), 4)])
@pytest.mark.parametrize("act", [1, 2])
def test_qgemm_act_matches_the_composition(mnk, wbits, act):
    M, N, K = mnk
    q = 127 if wbits == 8 else 7
    a, w = rand_codes((M, K), 127, 60), rand_codes((N, K), q, 61)
    ws = w if wbits == 8 else oracle.pack4(w)
    r = np.random.Generator(np.random.PCG64(62))
    sa = np.array([0.002], np.float32)
    sw = (r.random(N).astype(np.float32) + 0.5) * np.float32(1e-3)   # outputs of a few units: both GELU tails occur
    y_o, am_o = oracle.qgemm_act(a, ws, sa, sw, act, wbits, oracle.PER_ROW)
    for mk in (dev, dev_misaligned):
        y, am = mpq.qgemm_act(mk(a), mk(ws), dev(sa), dev(sw), act, wbits, mpq.PER_ROW)
        y_h = host(y)
        if act == 1:   # ReLU of a value that agrees to 1e-5 relative
            np.testing.assert_allclose(y_h, y_o, rtol=RTOL_Y, atol=0)
        else:          # GELU with the fp32 erf: relative, except in the negative tail where 1 + erf cancels
            pre, _ = oracle.qgemm(a, ws, sa, sw, wbits, oracle.PER_ROW)
            assert (np.abs(y_h - y_o) <= 2e-5 * np.abs(y_o) + 2e-7 * np.abs(pre)).all()
        # the absmax is exact for the values the kernel itself wrote, and within tolerance of the oracle's
        assert host(am)[0] == np.abs(y_h).max()
        assert host(am)[0] == pytest.approx(am_o[0], rel=2e-5)
    # running maximum over two calls
    am = dev(np.array([1e30], np.float32))
    mpq.qgemm_act(dev(a), dev(ws), dev(sa), dev(sw), act, wbits, mpq.PER_ROW, absmax=am, accumulate=True)
    assert host(am)[0] == np.float32(1e30)
    y, none = mpq.qgemm_act(dev(a), dev(ws), dev(sa), dev(sw), act, wbits, mpq.PER_ROW, want_absmax=False)
    assert none is None
    np.testing.assert_array_equal(host(y), host(mpq.qgemm_act(dev(a), dev(ws), dev(sa), dev(sw), act, wbits, mpq.PER_ROW)[0]))


# ------------------------------------------------------- qgemm + activation + Eq. 1 in the epilogue
@pytest.mark.parametrize("mnk,wbits", [((64, 256, 256), 8), ((33, 31, 130), 8), ((300, 70, 48), 4), ((2048, 2048, 384), 8),
                                        ((4100, 4092, 160), 4), ((2085, 2046, 112), 8), ((6272, 256, 512), 4),
                                        ((12288, 768, 128), 4), ((130, 70, 1296), 8), ((100, 200, 2080), 4)])
@pytest.mark.parametrize("act,bits", [(0, 8), (1, 8), (1, 4), (2, 8), (2, 4), (2, 2)])
def test_qgemm_act_codes_are_the_fake_quant_codes_of_the_activated_output(mnk, wbits, act, bits):
    """Two passes over the product: the calibration-only pass must find the absmax the storing pass
    finds, and the codes pass must give bit for bit what Eq. 1 gives on the fp32 output.  The oracle
    quantizes the GPU's own fp32 output (a stage of a chain is checked on the stage's own input);
    against the oracle's end-to-end composition codes may differ only where the pre-rounding value
    sits on a rounding boundary within the layer output's tolerance."""
    M, N, K = mnk
    q = 127 if wbits == 8 else 7
    a, w = rand_codes((M, K), 127, 70), rand_codes((N, K), q, 71)
    ws = w if wbits == 8 else oracle.pack4(w)
    r = np.random.Generator(np.random.PCG64(72))
    sa = np.array([0.002], np.float32)
    sw = (r.random(N).astype(np.float32) + 0.5) * np.float32(1e-3)
    for mk in (dev, dev_misaligned):
        da, dw, dsa, dsw = mk(a), mk(ws), dev(sa), dev(sw)
        y, am = mpq.qgemm_act(da, dw, dsa, dsw, act, wbits, mpq.PER_ROW)
        none, am_only = mpq.qgemm_act(da, dw, dsa, dsw, act, wbits, mpq.PER_ROW, want_y=False)
        assert none is None and host(am_only)[0] == host(am)[0]
        codes = host(mpq.qgemm_act_codes(da, dw, dsa, dsw, act, am, bits, wbits, mpq.PER_ROW))
        y_h, am_h = host(y), host(am)
        _, want, _ = oracle.fake_quant(y_h, am_h, bits)
        np.testing.assert_array_equal(codes, want)
    # end to end against the oracle alone
    y_o, am_o = oracle.qgemm_act(a, ws, sa, sw, act, wbits, oracle.PER_ROW)
    _, want_o, _ = oracle.fake_quant(y_o, am_o, bits)
    diff = codes.astype(np.int32) - want_o
    if diff.any():
        _, inv = oracle.bit_constants(float(am_o[0]), bits)
        p = y_o.astype(np.float64) * float(inv)
        off_boundary = np.abs(p - np.floor(p) - 0.5)
        bad = diff != 0
        assert np.abs(diff).max() <= 1
        assert (off_boundary[bad] <= 1e-4 * np.maximum(1.0, np.abs(p[bad]))).all()
        assert bad.mean() < 1e-3
    # a foreign absmax smaller than the data saturates at +-qmax; zero gives zero codes
    small = dev(np.array([am_h[0] / 4], np.float32))
    sat = host(mpq.qgemm_act_codes(dev(a), dev(ws), dev(sa), dev(sw), act, small, bits, wbits, mpq.PER_ROW))
    _, want_sat, _ = oracle.fake_quant(y_h, host(small), bits)
    np.testing.assert_array_equal(sat, want_sat)
    qmax = (1 << (bits - 1)) - 1
    assert sat.max() <= qmax and sat.min() >= -qmax
    zero = host(mpq.qgemm_act_codes(dev(a), dev(ws), dev(sa), dev(sw), act, dev(np.zeros(1, np.float32)), bits, wbits, mpq.PER_ROW))
    assert not zero.any()


# ---------------------------------------------------------------------------------- sse pair
@pytest.mark.parametrize("n", [1, 7, 4096, 100003, 1 << 20])
def test_sse_pair(n):
    r = np.random.Generator(np.random.PCG64(14))
    a = r.standard_normal(n).astype(np.float32)
    b = (a + 0.01 * r.standard_normal(n)).astype(np.float32)
    want = oracle.sse_pair(a, b)
    for mk in (dev, dev_misaligned):
        got = host(mpq.sse_pair(mk(a), mk(b)))[0]
        assert got == pytest.approx(want, rel=RTOL_SSE)
    assert host(mpq.sse_pair(dev(a), dev(a)))[0] == 0.0


def test_workspace_needs_no_initialisation_and_is_reusable():
    """One workspace serves call after call, whatever it holds on entry."""
    ws = mpq.Workspace()
    ws.get(1 << 20)
    x = data((700, 1028), 40)
    y = (x + 0.01).astype(np.float32)
    dx, dy = dev(x), dev(y)
    for fill in (0xFF, 0x00, 0xAB):
        ws.buf[:] = fill
        am = mpq.calibrate_absmax(dx, ws=ws)
        np.testing.assert_array_equal(host(am), oracle.absmax(x))
        np.testing.assert_allclose(host(mpq.quant_error(dx, am, ws=ws)), oracle.quant_error(x, oracle.absmax(x)),
                                   rtol=RTOL_SSE)
        assert host(mpq.sse_pair(dx, dy, ws=ws))[0] == pytest.approx(oracle.sse_pair(x, y), rel=RTOL_SSE)


# ------------------------------------------------------------------ configuration 1 end to end
def test_config1_whole_path():
    x, w = workloads.cfg1_tensors(0)
    dx, dw = dev(x), dev(w)
    mx, mw = mpq.calibrate_absmax(dx), mpq.calibrate_absmax(dw)
    mx_o, mw_o = oracle.absmax(x), oracle.absmax(w)
    np.testing.assert_array_equal(host(mx), mx_o)
    np.testing.assert_array_equal(host(mw), mw_o)
    for t, dt, m, dm in ((x, dx, mx_o, mx), (w, dw, mw_o, mw)):
        np.testing.assert_allclose(host(mpq.quant_error(dt, dm)), oracle.quant_error(t, m), rtol=RTOL_SSE)
        for b in range(2, 9):
            y_o, c_o, _ = oracle.fake_quant(t, m, b)
            y, c, _ = mpq.fake_quant(dt, dm, b, want_codes=True)
            np.testing.assert_array_equal(host(c), c_o)
            np.testing.assert_allclose(host(y), y_o, rtol=RTOL_Y, atol=0)
    np.testing.assert_array_equal(host(mpq.noise_inject(dw, mw, 4, 0.28867513, 0, 1)),
                                  oracle.noise_inject(w, mw_o, 4, 0.28867513, 0, 1))
    # (W8, A8) and (W4, A8), per-tensor scales
    _, ca, _ = mpq.fake_quant(dx, mx, 8, want_y=False, want_codes=True)
    sa = mpq.scale_from_absmax(mx, 8)
    _, ca_o, _ = oracle.fake_quant(x, mx_o, 8)
    for wb in (8, 4):
        _, cw, pw = mpq.fake_quant(dw, mw, wb, want_y=False, want_codes=wb == 8, want_packed4=wb == 4)
        _, cw_o, pw_o = oracle.fake_quant(w, mw_o, wb, want_packed4=wb == 4)
        sw = mpq.scale_from_absmax(mw, wb)
        y, acc = mpq.qgemm(ca, cw if wb == 8 else pw, sa, sw, wb, want_acc=True)
        y_o, acc_o = oracle.qgemm(ca_o, cw_o if wb == 8 else pw_o, oracle.scale_from_absmax(mx_o, 8),
                                  oracle.scale_from_absmax(mw_o, wb), wb)
        np.testing.assert_array_equal(host(acc), acc_o)
        np.testing.assert_allclose(host(y), y_o, rtol=RTOL_Y, atol=0)
        ref = x.astype(np.float64) @ w.astype(np.float64).T
        assert np.linalg.norm(host(y) - ref) / np.linalg.norm(ref) < (0.02 if wb == 8 else 0.25)
